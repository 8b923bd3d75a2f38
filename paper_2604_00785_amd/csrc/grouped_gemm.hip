// Stage 4 of Algorithm 1 (the three Grouped_mm calls around Silu(gate)*up) and
// its derivative, as grouped bf16 MFMA GEMMs: one launch covers every expert.
//
// One workgroup of FOUR waves (one per SIMD, 512 registers each) computes one 256x256 output tile
// with a 64-deep K step; the waves form a 2 x 2 grid and each owns a 128x128 piece = 8x8
// v_mfma_f32_16x16x32_bf16 accumulators, which live in the 256 accumulation registers.  Against
// eight waves with 128x64 pieces this reads a third less operand data out of LDS per FLOP, and the
// 16x16x32 form draws less power per FLOP than the 32x32x16 form (the chip is power-limited on
// real data), but with one wave per SIMD nothing covers a wave's own stalls, so the main loop is
// written instruction by instruction:
//   * MFMAs, LDS fragment reads and direct-to-LDS loads are inline assembly in program order; the
//     accumulators are pinned to accumulation registers, so the compiler has nothing to move;
//   * between two MFMAs there is at most one other instruction (a fragment read, or a load);
//   * no vector-ALU instruction and no branch inside a K step: loads use a scalar base that is
//     advanced by scalar adds plus a 32-bit lane offset computed once per tile; the eight loads a
//     wave issues per operand tile share one M0 value (the instruction's immediate offset moves
//     the LDS address; the lane offset takes the same amount out of the global address again);
//   * the last three K steps of a tile (the last one that loads, which is the one that may load a
//     partial step of a weight gradient; the one that only awaits; the last one) are separate copies
//     of the step, and a tile enters the ring of LDS slots at the phase that puts those three on
//     phases 0, 1 and 2.
//
// The two operand tiles of a step (32 KB each) live in a ring of five LDS slots (160 KB, all
// there is): A(t) in slot 2t mod 5, B(t) in slot (2t+1) mod 5, so two and a half steps are
// resident.  Step t loads A(t+2) during its first 32-deep sub-step, into the slot B(t-1) left;
// its barrier follows that sub-step: behind it the tiles of step t+1 are complete (the wave's own
// loads of A(t+2) may still be in flight) and every wave is done with A(t), whose slot B(t+2) is
// loaded into during the second sub-step.  Fragments are double-buffered in registers: the reads
// of the next sub-step are issued between the MFMAs of the current one.
//
// Tile layouts.  An operand that is contiguous along K in memory (activations [rows, K],
// forward weights [N, K]) is kept as [256 rows][64 k] with 128-byte rows whose eight 16-byte
// pieces are rotated by the row (fragment = one ds_read_b128 per lane); the swizzle is
// applied on the global side of the fill, since a direct-to-LDS load writes LDS linearly.  An
// operand that is contiguous along its other dimension (weights in dgrad, both operands in
// wgrad) is kept as it lies in memory, [64 k][256 n] with 512-byte rows, and read with the
// transposing LDS load ds_read_b64_tr_b16, two per fragment (it moves half the bytes per cycle
// of ds_read_b128, which makes the weight gradients LDS-bound).
//
// The MFMAs are issued as (weight fragment) x (activation fragment), so a lane ends up with
// four consecutive output COLUMNS of one row.  The epilogue reads the accumulators by hand, rounds
// to bf16, stages 16 or 32 rows of the wave's 128x128 piece at a time in the wave's own 8 KB of LDS
// and writes them out in full 256-byte row segments; the SwiGLU forward and backward formulas are
// applied on the way, on the fp32 accumulators.
//
// Tiles of the row-grouped products are found on the device from expert_offsets: every wave
// turns the tile number into (expert, first row, column tile); inside an expert the row tiles are
// innermost; experts without rows own no tile; rows past an expert's end are clamped on load and
// masked on store, and 32-row groups without a valid row issue no MFMA.
#include <type_traits>
#include <utility>
#include "common.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 256;
constexpr int TILE_BYTES = BM * BK * 2;               // one operand tile (32 KB)
constexpr int NSLOT = 5;                              // ring of operand tile slots
constexpr int LDS_BYTES = NSLOT * TILE_BYTES;         // 160 KB: everything a workgroup can have
constexpr int LOAD_BIAS = 4096;                       // see dma16_imm
constexpr int slot_of_a(int p) { return (2 * p) % NSLOT; }       // p = ring phase of the step
constexpr int slot_of_b(int p) { return (2 * p + 1) % NSLOT; }

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int N> using IC = std::integral_constant<int, N>;
template <typename F, int... I> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(IC<I>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

enum GemmMode { GATE_UP = 0, DOWN = 1, DGRAD_H = 2, DGRAD_X = 3, WGRAD = 4, WGRAD_GATHER = 5, DGRAD_H_GATE = 6,
                WGRAD_GATHER_A = 7 };
// WGRAD_GATHER / WGRAD_GATHER_A: a weight gradient whose B / A operand rows are token rows found through
// row_token.  DGRAD_H_GATE: DGRAD_H for a forward pass that folded the gate weight into h: its A rows are
// rows of dout found through row_token, its epilogue scales by the row's gate weight and also emits the
// row's partial dot product with h = silu(g) u (the gradient of the gate weight).
constexpr bool is_wgrad(int mode) { return mode == WGRAD || mode == WGRAD_GATHER || mode == WGRAD_GATHER_A; }
constexpr bool is_dgrad_h(int mode) { return mode == DGRAD_H || mode == DGRAD_H_GATE; }

struct GemmArgs {
  // row-grouped products (modes 0-3, 6)
  const uint16_t* A0;   // [R_cap, K]   activations (phase 0)
  const uint16_t* A1;   // second K phase of DGRAD_X (du), else unused
  const uint16_t* B0;   // weights, stacked over experts
  const uint16_t* B1;   // Wu (GATE_UP: the up half of the column tile; DGRAD_X: second K phase)
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
  int K;                // reduction length of one phase (row-grouped products)
  int N;                // output columns (per half for GATE_UP)
  int n_tiles;          // column tiles
  int m_tiles_cap;      // upper bound on row tiles (row-grouped products); row tiles of one dW (WGRAD)
  // WGRAD: out[e][M][N] = sum over the expert's rows of A[r][M] * B[r][N]
  int M;
};

// 512 bytes of zeros: what the reduction rows past an expert's end read in the weight-gradient products.
__device__ __attribute__((aligned(512))) uint32_t g_zero_block[128];

// [256 rows][64 k] tile, 128-byte rows: the 16-byte piece `logical` (0..7) of `row` lies at physical piece
// (logical + row) mod 8.  A fragment read (16 rows x 4 neighbouring pieces per instruction) then costs 8.5
// cycles per CU, as a linear read does; XOR-ing the piece with (row ^ row >> 3) & 7 costs 8.9, no swizzle 16.
// This is the inverse: which logical piece a fill has to fetch for physical piece `phys`.
__device__ __forceinline__ int kc_logical_piece(int row, int phys) { return (phys - row) & 7; }
// [64 k][256 n] tile: 16-byte pieces of a k row are XOR-swizzled with 4*(k & 3), which spreads the
// four k rows that 16 lanes of a transposing read touch over four different 64-byte bank groups.
__device__ __forceinline__ int kn_piece(int krow, int piece) { return piece ^ ((krow & 3) << 2); }

// Everything the main loop issues is inline assembly in program order (asm volatile statements keep
// their order), with immediate offsets, and is awaited by hand: fragments are read one sub-step
// ahead and loads several steps ahead, which the compiler's own wait insertion cannot express.
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
// Direct-to-LDS loads, 16 bytes per lane: lane l lands at M0 + OFF + 16 l, and reads global address
// (scalar base) + (32-bit lane offset) + OFF.  The immediate moves both addresses: a wave's eight loads
// of a tile use OFF = (i - 4) * 1024 with one M0 value, their lane offsets carry -OFF, and LOAD_BIAS
// (subtracted from the scalar base, added to every lane offset) keeps the lane offsets non-negative.
// Nothing else in this file uses M0.
template <int OFF> __device__ __forceinline__ void set_m0(uint32_t lds_base) {
  asm volatile("s_add_i32 m0, %0, %1" :: "s"(lds_base), "n"(OFF) : "memory", "scc");
}
__device__ __forceinline__ void set_m0_rt(uint32_t lds_addr) { asm volatile("s_mov_b32 m0, %0" :: "s"(lds_addr) : "memory"); }
template <int OFF> __device__ __forceinline__ void dma16_imm(uint32_t voff, const char* sbase) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" :: "v"(voff), "s"(sbase), "n"(OFF) : "memory");
}
// the same with a 64-bit address per lane (used once per tile at most, for rows past an expert's end)
template <int OFF> __device__ __forceinline__ void dma16_lane_imm(const char* p) {
  asm volatile("global_load_lds_dwordx4 %0, off offset:%1" :: "v"(p), "n"(OFF) : "memory");
}
// A 4-byte load as (scalar base) + (32-bit lane offset) + immediate, awaited by hand like the loads above.
template <int OFF> __device__ __forceinline__ int load_i32(uint32_t voff, const int32_t* sbase) {
  int v;
  asm volatile("global_load_dword %0, %1, %2 offset:%3" : "=v"(v) : "v"(voff), "s"(sbase), "n"(OFF) : "memory");
  return v;
}
template <int N> __device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }
template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wg_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

// A fragment of a [64 k][256 n] tile: two transposing reads (k rows +0..3 and +4..7 of the lane's column).
union KnFrag {
  s16x4 h[2];
  bf16x8_t v;
};

// sigmoid through the hardware exp2 and reciprocal (each about 1 ulp): far inside bf16 rounding.
// exp2 overflows to +inf for very negative g and the reciprocal then returns 0, as it should.
__device__ __forceinline__ float sigmoid_f(float g) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
}
__device__ __forceinline__ float silu_f(float g) { return g * sigmoid_f(g); }

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
//
// With at most 128 experts (two per lane) the experts are not listed in index order: those whose tile count
// is a whole number of XCD runs come first, then those that fill half a run, then the rest.  The first
// two groups then start on run boundaries, so such an expert's tiles are worked on by one XCD at one
// time and its activation rows are fetched into one L2 once; an expert that straddles two runs has its
// rows fetched by both.  The lane keeps its expert's row range and first list position for the whole
// kernel, so the lookup needs no memory access (which would otherwise sit in front of every tile's
// first loads) and no scan.
// (kept as six plain registers: a struct of arrays behind a reference ends up in scratch memory)
__device__ __forceinline__ void sorted_first_tiles(int tiles0, int tiles1, int run, int lane, int& first0, int& first1) {
  const int r0 = tiles0 % run, r1 = tiles1 % run;
  const int cls0 = r0 == 0 ? 0 : (2 * r0 == run ? 1 : 2);
  const int cls1 = r1 == 0 ? 0 : (2 * r1 == run ? 1 : 2);
  int base = 0;
  first0 = 0;
  first1 = 0;
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const int mine0 = cls0 == c ? tiles0 : 0;
    const int inc0 = wave_incl_scan(mine0, lane);
    if (cls0 == c) first0 = base + inc0 - mine0;
    base += __shfl(inc0, 63, 64);
    const int mine1 = cls1 == c ? tiles1 : 0;
    const int inc1 = wave_incl_scan(mine1, lane);
    if (cls1 == c) first1 = base + inc1 - mine1;
    base += __shfl(inc1, 63, 64);
  }
}
constexpr int LANE_EXPERTS_MAX = 128;
// One half (experts 64 h .. 64 h + 63, one per lane) of the register-resident lookup.
__device__ __forceinline__ bool find_tile_half(int h, int lo, int hi, int first, int n_tiles, int tile, int& e, int& m0,
                                               int& m_end, int& nt) {
  const int row_tiles = (hi - lo + BM - 1) / BM;
  const int tiles = row_tiles * n_tiles;
  const unsigned long long hit = __ballot(tiles > 0 && first <= tile && tile < first + tiles);
  if (!hit) return false;
  const int l = __ffsll(hit) - 1;
  e = h * 64 + l;
  const int q = tile - __shfl(first, l, 64);
  const int rt = __shfl(row_tiles, l, 64);
  nt = q / rt;
  m0 = __shfl(lo, l, 64) + (q - nt * rt) * BM;
  m_end = __shfl(hi, l, 64);
  return true;
}
__device__ __forceinline__ void find_tile(const int32_t* offsets, int E, int lo0, int hi0, int first0, int lo1, int hi1,
                                          int first1, int n_tiles, int tile, int lane, int& e, int& m0, int& m_end, int& nt) {
  e = 0; m0 = 0; m_end = 0; nt = 0;
  if (E <= LANE_EXPERTS_MAX) {
    if (find_tile_half(0, lo0, hi0, first0, n_tiles, tile, e, m0, m_end, nt)) return;
    find_tile_half(1, lo1, hi1, first1, n_tiles, tile, e, m0, m_end, nt);
    return;
  }
  int base = 0;
  for (int e0 = 0; e0 < E; e0 += 64) {
    const int ee = e0 + lane;
    const int lo = ee < E ? offsets[ee] : 0, hi = ee < E ? offsets[ee + 1] : 0;
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
// registers across the main loop.
typedef const __attribute__((address_space(4))) GemmArgs* ArgPtr;
template <int ARG> __device__ __forceinline__ ArgPtr reload_args() {   // ARG: which of the kernel's GemmArgs
  ArgPtr p = (ArgPtr)__builtin_amdgcn_kernarg_segment_ptr() + ARG;
  asm volatile("" : "+s"(p));
  return p;
}

// A wave-uniform pointer as two scalar registers.  readfirstlane returns a signed int: it is widened
// through uint32_t, or a set bit 31 of the low half would smear into the high half.
__device__ __forceinline__ const char* scalarize(const char* p) {
  const uint64_t u = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u)));
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u >> 32)));
  return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | static_cast<uint64_t>(lo));
}

// What a workgroup knows about one tile: where it lies, where its operand loads come from, how many
// K steps it has.
struct TileState {
  int e, m0, m_end, nt, n0;     // expert, first output row, end of the valid rows, column tile, first output column
  int nv;                       // 32-row groups of this wave's 128 rows that hold a valid row
  bool second;                  // tile of the second weight gradient of a pair
  int nk, nk_phase;             // K steps in total / in the first K phase
  int nmain, p0;                // steps in front of the last three; ring phase of step 0
  int k_lo, k_hi;               // weight gradients: the expert's row range is the reduction
  bool last_partial;            // weight gradients: the last step holds fewer than 64 rows
  uint32_t voa[8], vob[8];      // lane offsets of the eight loads per operand tile, in bytes
  uint32_t vcb[8];              // gathered operand: lane offset of a load without its token row
  int tokn[8], tokn1[8];        // gathered operand: tokens of the lane's eight reduction rows of coming steps
  const char* sa_next;          // scalar bases of the next A / B tile to load (LOAD_BIAS low)
  const char* sb_next;
  const char* sa_phase1;        // DGRAD_X: bases of the second K phase
  const char* sb_phase1;
  size_t a_step, b_step;        // bytes per step
  const int32_t* row_tok;       // gathered operand: token of the expert's first reduction row onwards
};

// One product's tile list, walked by this workgroup from list position first_tile in steps of
// gridDim.x.  Returns the position at which the workgroup left the list, counted from its end:
// where it enters a list that follows in the same launch.
template <int MODE, int ARG>
__device__ __forceinline__ int gemm_tile_list(const GemmArgs& a, int first_tile) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  constexpr bool A_KN = is_wgrad(MODE);                                           // stored [k][m]
  constexpr bool B_KN = (is_wgrad(MODE) || is_dgrad_h(MODE) || MODE == DGRAD_X);  // stored [k][n]
  constexpr bool GATHER_B = (MODE == WGRAD_GATHER);
  constexpr bool GATHER_A = (MODE == WGRAD_GATHER_A);

  // ---------------- tile list ---------------------------------------------------
  int total;
  // experts `lane` and `lane + 64`: row range and list position of the first tile, kept for the whole kernel
  // when E <= LANE_EXPERTS_MAX
  int lo0 = 0, hi0 = 0, first0 = 0, lo1 = 0, hi1 = 0, first1 = 0;
  // WGRAD / WGRAD_GATHER with a second A operand (A1 -> O1): two weight gradients that share their B
  // operand in one launch; an expert's tiles of the first come before its tiles of the second
  int wpair = 1;
  if constexpr (MODE == WGRAD_GATHER || MODE == WGRAD) wpair = a.A1 != nullptr ? 2 : 1;
  if constexpr (is_wgrad(MODE)) {
    total = a.E * a.m_tiles_cap * a.n_tiles * wpair;
  } else {
    total = count_row_tiles(a.offsets, a.E, tid0 & 63) * a.n_tiles;
    if (a.E <= LANE_EXPERTS_MAX) {
      const int e0 = tid0 & 63, e1 = 64 + (tid0 & 63);
      if (e0 < a.E) { lo0 = a.offsets[e0]; hi0 = a.offsets[e0 + 1]; }
      if (e1 < a.E) { lo1 = a.offsets[e1]; hi1 = a.offsets[e1 + 1]; }
      sorted_first_tiles((hi0 - lo0 + BM - 1) / BM * a.n_tiles, (hi1 - lo1 + BM - 1) / BM * a.n_tiles, gridDim.x >> 3,
                         tid0 & 63, first0, first1);
    }
  }
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<size_t>(LDS_PTR(lds)));
  // M0 base of this wave's loads: the middle of its 8 KB share of tile slot 0 (immediates reach -4096 .. +3072)
  const uint32_t lds_fill = __builtin_amdgcn_readfirstlane(lds0 + wave * 8192 + 4096);

  const int lane = tid0 & 63;
  // Everything about tile number `tile` of the list that does not depend on the K step.
  auto setup_tile = [&](int tile, TileState& t) __attribute__((always_inline)) {
  // the thread id is laundered per tile so that the lane-dependent pieces of the load offsets are recomputed for
  // every tile instead of staying live (and spilling) across the main loop
  int tid = tid0;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  int e, m0, m_end, nt;
  bool second = false;
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
    find_tile(a.offsets, a.E, lo0, hi0, first0, lo1, hi1, first1, a.n_tiles, tile, lane, e, m0, m_end, nt);
    nt = __builtin_amdgcn_readfirstlane(nt);
  }
  // tile coordinates are wave-uniform: keep them in scalar registers, so that everything derived
  // from them (operand base addresses in particular) is scalar too
  e = __builtin_amdgcn_readfirstlane(e);
  m0 = __builtin_amdgcn_readfirstlane(m0);
  m_end = __builtin_amdgcn_readfirstlane(m_end);
  const int n0 = nt * (MODE == GATE_UP ? BN / 2 : BN);
  t.e = e; t.m0 = m0; t.m_end = m_end; t.nt = nt; t.n0 = n0; t.second = second;
  // 32-row groups of this wave's 128 rows that hold at least one valid row (the others issue no MFMA)
  int nv = 4;
  if constexpr (!is_wgrad(MODE)) {
    nv = (m_end - m0 - wm * 128 + 31) >> 5;
    nv = nv < 0 ? 0 : (nv > 4 ? 4 : nv);
    nv = __builtin_amdgcn_readfirstlane(nv);
  }
  t.nv = nv;

  // ---------------- operand sources -------------------------------------------
  // Per K step and operand tile a wave issues eight direct-to-LDS loads of 1 KB each:
  //  K-contiguous source ([row][k]): load i of wave w fills tile rows 64 w + 8 i .. + 8;
  //    lane l -> row + l/8, physical piece l%8, i.e. logical piece kc_logical_piece(row, l%8).
  //    The base advances by 64 elements per step.
  //  n-contiguous source ([k][n]): load i of wave w fills k rows 2 (8 w + i), + 1;
  //    lane l -> k row + l/32, physical piece l%32 = logical piece kn_piece(k row, l%32).
  //    The base advances by 64 rows per step.
  // Lane offsets carry LOAD_BIAS - (i - 4) * 1024 (see dma16_imm); the scalar bases lie LOAD_BIAS low.
  uint32_t (&voa)[8] = t.voa;           // lane offsets in bytes
  uint32_t (&vob)[8] = t.vob;
  const char* abase;                    // step 0 of phase 0, without the bias
  const char* bbase;
  ptrdiff_t a_phase = 0, b_phase = 0;   // byte offset of the second K phase (DGRAD_X)
  size_t a_step, b_step;                // bytes per step
  int k_lo = 0, k_hi = 0;               // WGRAD: the expert's row range is the reduction
  const int32_t* row_tok = nullptr;     // GATHER_A/B: token of the expert's first reduction row onwards
  uint32_t (&vcb)[8] = t.vcb;           // GATHER_A/B: lane offset of a load without its token row
#pragma unroll
  for (int i = 0; i < 8; ++i) { t.vcb[i] = 0; t.tokn[i] = 0; t.tokn1[i] = 0; }
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
    for (int i = 0; i < 8; ++i) {
      const int krow = (wave * 8 + i) * 2 + (lane >> 5);
      const int piece = kn_piece(krow, lane & 31);
      int ca = piece * 8;  if (m0 + ca > a.M - 8) ca = a.M - 8 - m0;
      int cb = piece * 8;  if (n0 + cb > a.N - 8) cb = a.N - 8 - n0;
      const uint32_t fix = static_cast<uint32_t>(LOAD_BIAS - (i - 4) * 1024);
      voa[i] = static_cast<uint32_t>((krow * a.M + ca) * 2) + fix;
      vob[i] = static_cast<uint32_t>((krow * a.N + cb) * 2) + fix;
      if constexpr (GATHER_B) vcb[i] = static_cast<uint32_t>(cb * 2) + fix;
      if constexpr (GATHER_A) vcb[i] = static_cast<uint32_t>(ca * 2) + fix;
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
    for (int i = 0; i < 8; ++i) {
      const int row = (wave * 8 + i) * 8 + (lane >> 3);
      const int chunk = kc_logical_piece(row, lane & 7);
      int r = row;
      if (m0 + r > m_end - 1) r = m_end - 1 - m0;
      const uint32_t fix = static_cast<uint32_t>(LOAD_BIAS - (i - 4) * 1024);
      if (gathered) voa[i] = (static_cast<uint32_t>(a.row_token[m0 + r]) * a.K + chunk * 8) * 2u + fix;
      else voa[i] = static_cast<uint32_t>((r * a.K + chunk * 8) * 2) + fix;
    }
    if constexpr (MODE == DGRAD_X) { a_phase = (a.A1 - a.A0) * 2; nk *= 2; }
    const size_t wsz = static_cast<size_t>(a.N) * a.K;
    if constexpr (!B_KN) {
      // GATE_UP: a wave's 128 tile rows are 64 rows of Wg and the same 64 rows of Wu: tile rows
      // [0,64) Wg n0.., [64,128) Wu n0.., [128,192) Wg n0+64.., [192,256) Wu n0+64.. (wave w fills its own 64)
      const uint16_t* w = a.B0;
      int first_col = wave * 64;
      if constexpr (MODE == GATE_UP) {
        if (wave & 1) w = a.B1;
        first_col = (wave >> 1) * 64;
      }
      bbase = reinterpret_cast<const char*>(w + static_cast<size_t>(e) * wsz + static_cast<size_t>(n0) * a.K);
      b_step = BK * 2;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = (wave * 8 + i) * 8 + (lane >> 3);   // LDS row of the B tile
        const int chunk = kc_logical_piece(row, lane & 7);
        int col = first_col + i * 8 + (lane >> 3);
        if (n0 + col > a.N - 1) col = a.N - 1 - n0;
        vob[i] = static_cast<uint32_t>((col * a.K + chunk * 8) * 2) + static_cast<uint32_t>(LOAD_BIAS - (i - 4) * 1024);
      }
    } else {  // DGRAD_H / DGRAD_X: weights stored [K][N]
      bbase = reinterpret_cast<const char*>(a.B0 + static_cast<size_t>(e) * wsz + n0);
      b_step = static_cast<size_t>(BK) * a.N * 2;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int krow = (wave * 8 + i) * 2 + (lane >> 5);
        int cb = kn_piece(krow, lane & 31) * 8;
        if (n0 + cb > a.N - 8) cb = a.N - 8 - n0;
        vob[i] = static_cast<uint32_t>((krow * a.N + cb) * 2) + static_cast<uint32_t>(LOAD_BIAS - (i - 4) * 1024);
      }
      if constexpr (MODE == DGRAD_X) b_phase = (a.B1 - a.B0) * 2;
    }
  }

  // Both bases live in scalar registers and are advanced by scalar adds: steps are loaded in order.
  t.sa_next = scalarize(abase - LOAD_BIAS);
  t.sb_next = scalarize(bbase - LOAD_BIAS);
  t.sa_phase1 = nullptr;
  t.sb_phase1 = nullptr;
  if constexpr (MODE == DGRAD_X) { t.sa_phase1 = scalarize(abase + a_phase - LOAD_BIAS); t.sb_phase1 = scalarize(bbase + b_phase - LOAD_BIAS); }
  t.a_step = a_step; t.b_step = b_step; t.k_lo = k_lo; t.k_hi = k_hi; t.row_tok = row_tok; t.nk = nk; t.nk_phase = nk_phase;
  t.last_partial = is_wgrad(MODE) && ((k_hi - k_lo) % BK) != 0;
  // The last three steps of a tile are copies of their own: the last step that loads (it loads the tile's last
  // step, the one that may be partial in a weight gradient), the step that only awaits, and the last one.
  // The tile enters the ring at the phase p0 that puts these three on phases 0, 1 and 2, so that the steps
  // before them end on a round of the five phases.
  t.nmain = nk >= 3 ? nk - 3 : 0;
  t.p0 = nk >= 3 ? (NSLOT - t.nmain % NSLOT) % NSLOT : (nk == 2 ? 1 : 2);
  };


  // Load i of the A / B tile of step kt (M0 must point at the tile's slot already).  In the weight gradients the
  // last step of an expert may be partial (its row count is no multiple of 64): reduction rows at or past the
  // expert's end then read zeros in one operand (per-lane 64-bit addresses) and a valid row in the other.
  // SP 0: the step is known to be whole; 1: known to be the partial one; 2: look (first loads of a tile).
  auto a_part = [&](TileState& t, int kt, auto i_tag, auto sp_tag) __attribute__((always_inline)) {
    constexpr int i = decltype(i_tag)::value, SP = decltype(sp_tag)::value;
    constexpr int OFF = (i - 4) * 1024;
    if constexpr (is_wgrad(MODE) && !GATHER_A && SP != 0) {
      if (SP == 1 || (t.last_partial && kt == t.nk - 1)) {
        const int krow = t.k_lo + kt * BK + (wave * 8 + i) * 2 + (lane >> 5);
        dma16_lane_imm<OFF>(krow < t.k_hi ? t.sa_next + t.voa[i]
                                        : reinterpret_cast<const char*>(g_zero_block) + (lane & 31) * 16 - OFF);
        return;
      }
    }
    dma16_imm<OFF>(t.voa[i], t.sa_next);   // GATHER_A: rows past the expert's end were clamped when their tokens were fetched
  };
  auto b_part = [&](TileState& t, int kt, auto i_tag, auto sp_tag) __attribute__((always_inline)) {
    constexpr int i = decltype(i_tag)::value, SP = decltype(sp_tag)::value;
    constexpr int OFF = (i - 4) * 1024;
    if constexpr ((GATHER_A || MODE == WGRAD) && SP != 0) {
      if (SP == 1 || (t.last_partial && kt == t.nk - 1)) {
        const int krow = t.k_lo + kt * BK + (wave * 8 + i) * 2 + (lane >> 5);
        if constexpr (GATHER_A) {
          // the gathered operand repeats the expert's last row past its end: this one reads zeros there
          dma16_lane_imm<OFF>(krow < t.k_hi ? t.sb_next + t.vob[i]
                                          : reinterpret_cast<const char*>(g_zero_block) + (lane & 31) * 16 - OFF);
        } else {
          // ... and the other operand reads its last valid row there, so that zero times it is zero
          dma16_lane_imm<OFF>(t.sb_next + t.vob[i] - (krow < t.k_hi ? 0 : static_cast<size_t>(krow - (t.k_hi - 1)) * a.N * 2));
        }
        return;
      }
    }
    dma16_imm<OFF>(t.vob[i], t.sb_next);   // GATHER_B: rows past the expert's end were clamped when their tokens were fetched
  };
  auto a_end = [&](TileState& t, int kt) __attribute__((always_inline)) {
    t.sa_next += t.a_step;
    if constexpr (MODE == DGRAD_X) {
      if (kt + 1 == t.nk_phase) t.sa_next = t.sa_phase1;
    }
  };
  auto b_end = [&](TileState& t, int kt) __attribute__((always_inline)) {
    t.sb_next += t.b_step;
    if constexpr (MODE == DGRAD_X) {
      if (kt + 1 == t.nk_phase) t.sb_next = t.sb_phase1;
    }
  };
  // GATHER_A/B: the tokens of the lane's eight reduction rows of step kt (rows 2 (8 w + i) + lane / 32), loaded
  // without any vector-ALU work except in an expert's last, partial step (rows past its end repeat its last
  // row: the other operand is zero there), and their turn into lane offsets of the gathered operand's loads.
  // The loads are asynchronous: apply_tok may only run after a wait that covers them.
  const uint32_t tok_voff = static_cast<uint32_t>(((wave * 8) * 2 + (lane >> 5)) * 4);   // row of load 0; load i: + 2 i rows
  auto fetch_tok = [&](TileState& t, int kt, int (&tk)[8]) __attribute__((always_inline)) {
    if constexpr (GATHER_B || GATHER_A) {
      if (t.k_lo + (kt + 1) * BK > t.k_hi) {
        const int last = t.k_hi - t.k_lo - 1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          int r = kt * BK + (wave * 8 + i) * 2 + (lane >> 5);
          if (r > last) r = last;
          tk[i] = load_i32<0>(static_cast<uint32_t>(r) * 4u, t.row_tok);
        }
      } else {
        const int32_t* base = t.row_tok + static_cast<size_t>(kt) * BK;
        tk[0] = load_i32<0>(tok_voff, base);
        tk[1] = load_i32<8>(tok_voff, base);
        tk[2] = load_i32<16>(tok_voff, base);
        tk[3] = load_i32<24>(tok_voff, base);
        tk[4] = load_i32<32>(tok_voff, base);
        tk[5] = load_i32<40>(tok_voff, base);
        tk[6] = load_i32<48>(tok_voff, base);
        tk[7] = load_i32<56>(tok_voff, base);
      }
    }
  };
  auto apply_tok = [&](TileState& t, int (&tk)[8]) __attribute__((always_inline)) {
    if constexpr (GATHER_B || GATHER_A) {
      const uint32_t row_bytes = static_cast<uint32_t>(GATHER_B ? a.N : a.M) * 2u;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        asm volatile("" : "+v"(tk[i]));   // not before the wait that precedes this call
        const uint32_t off = static_cast<uint32_t>(tk[i]) * row_bytes + t.vcb[i];
        if constexpr (GATHER_B) t.vob[i] = off; else t.voa[i] = off;
      }
    }
  };

  // ---------------- fragment addresses ------------------------------------------
  // Slot, block and sub-step are immediate offsets of the LDS reads, which reach 64 KB: one set of
  // per-lane addresses serves slots 0-1, one slots 2-3, one slot 4; four addresses per set and operand.
  //  [row][k] tile: block b = rows 16 b + (lane & 15), sub-step s (32 k) = logical piece 4 s + lane / 16.
  //    The row's share of the swizzle is lane & 7 whatever the block, so the address of (b, s) is
  //    base[s] + 2048 b.
  //  [k][n] tile: block b = columns 16 b + (lane & 15); within 16 lanes, lane i supplies the address of four
  //    consecutive n of k row i / 4, n group i % 4, and lane l receives k rows 0..3 of column l; lanes
  //    16 g .. 16 g + 15 take k rows 8 g .. of the sub-step.  The k-row swizzle XORs bits 1-2 of the block
  //    number, so the address of block b is base[b / 2] + 32 (b & 1); the second half of a fragment lies
  //    4 k rows = 2048 bytes further, sub-step 1 32 k rows = 16384 bytes further.
  uint32_t fa_base[3][4], fb_base[3][4];
#pragma unroll
  for (int st = 0; st < 3; ++st) {
    const uint32_t org = lds0 + st * 2 * TILE_BYTES;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int i16 = lane & 15;
      // [row][k]
      const int pc = ((x & 1) * 4 + (lane >> 4) + (lane & 7)) & 7;   // sub-step x & 1; the block is an immediate offset
      const uint32_t kc_a = org + (wm * 128 + i16) * 128 + pc * 16;
      const uint32_t kc_b = org + (wn * 128 + i16) * 128 + pc * 16;
      // [k][n]
      const int krow = (lane >> 4) * 8 + (i16 >> 2);
      const int sw = krow & 3;
      const uint32_t kn_lane = krow * 512 + ((x ^ sw) << 6) + ((i16 >> 1) & 1) * 16 + (i16 & 1) * 8;
      const uint32_t kn_a = org + wm * 256 + kn_lane;
      const uint32_t kn_b = org + wn * 256 + kn_lane;
      fa_base[st][x] = A_KN ? kn_a : kc_a;
      fb_base[st][x] = B_KN ? kn_b : kc_b;
    }
  }

  // ---------------- main loop ----------------------------------------------------
  f32x4_t acc[8][8];

  // two fragment sets: one feeds the MFMAs while the other is being read
  KnFrag fa[2][8], fb[2][8];
  constexpr int A_OPS_PER_BLK = A_KN ? 2 : 1, B_OPS_PER_BLK = B_KN ? 2 : 1;
  // Read instruction number `op` of a sub-step: the A blocks first (only the live ones), then the B blocks.
  auto read_op = [&](auto slot_a_tag, auto slot_b_tag, auto s_tag, auto set_tag, auto nv_tag, auto op_tag) __attribute__((always_inline)) {
    constexpr int SA = decltype(slot_a_tag)::value, SB = decltype(slot_b_tag)::value, S = decltype(s_tag)::value;
    constexpr int SET = decltype(set_tag)::value, NV = decltype(nv_tag)::value, OP = decltype(op_tag)::value;
    constexpr int A_OPS = 2 * NV * A_OPS_PER_BLK;
    if constexpr (OP < A_OPS) {
      constexpr int blk = OP / A_OPS_PER_BLK;
      if constexpr (A_KN) {
        constexpr int half = OP % 2;
        fa[SET][blk].h[half] = lds_read_tr_b64<(SA & 1) * TILE_BYTES + S * 16384 + half * 2048 + (blk & 1) * 32>(fa_base[SA >> 1][blk >> 1]);
      } else {
        fa[SET][blk].v = lds_read_b128<(SA & 1) * TILE_BYTES + blk * 2048>(fa_base[SA >> 1][S]);
      }
    } else {
      constexpr int OB = OP - A_OPS;
      constexpr int blk = OB / B_OPS_PER_BLK;
      if constexpr (B_KN) {
        constexpr int half = OB % 2;
        fb[SET][blk].h[half] = lds_read_tr_b64<(SB & 1) * TILE_BYTES + S * 16384 + half * 2048 + (blk & 1) * 32>(fb_base[SB >> 1][blk >> 1]);
      } else {
        fb[SET][blk].v = lds_read_b128<(SB & 1) * TILE_BYTES + blk * 2048>(fb_base[SB >> 1][S]);
      }
    }
  };
  // weight fragment first: the lane then holds 4 consecutive output columns of one row
  auto mma = [&](auto set_tag, auto i_tag, auto j_tag) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value, i = decltype(i_tag)::value, j = decltype(j_tag)::value;
    f32x4_t& c = acc[i][j];
    const bf16x8_t& wfrag = fb[SET][j].v;
    const bf16x8_t& afrag = fa[SET][i].v;
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(wfrag), "v"(afrag));
  };

  // One 32-deep sub-step: the live MFMAs of fragment set SET, and between them (one per gap) the read
  // instructions of the next sub-step and, in a step that loads (LOADS), the wave's eight loads of one
  // tile.  Gap g is the place after MFMA g: reads take the even gaps 0, 2, .. (every gap when both operands
  // need two reads per block), M0 is set in gap 1, loads take gaps 3, 7, .., 31; what does not fit behind
  // the last live MFMA follows it.
  auto sub_step = [&](auto set_tag, auto nv_tag, auto nreads_tag, auto reader, auto loads_tag, auto set_m0_fn, auto loader)
      __attribute__((always_inline)) {
    constexpr int SET = decltype(set_tag)::value, NV = decltype(nv_tag)::value;
    constexpr int NREADS = decltype(nreads_tag)::value;
    constexpr bool LOADS = decltype(loads_tag)::value != 0;
    constexpr int ML = 16 * NV;                         // live MFMAs: blocks i < 2 NV, all j
    constexpr int RSTRIDE = NREADS > 32 ? 1 : 2;
    constexpr int LAST_GAP = (NREADS - 1) * RSTRIDE > 31 ? (NREADS - 1) * RSTRIDE : 31;
    constexpr int SLOTS = ML > LAST_GAP + 1 ? ML : LAST_GAP + 1;
    static_for<SLOTS>([&](auto g_tag) {
      constexpr int g = decltype(g_tag)::value;
      if constexpr (g < ML) mma(IC<SET>{}, IC<g / 8>{}, IC<g % 8>{});
      if constexpr (g % RSTRIDE == 0 && g / RSTRIDE < NREADS) reader(IC<g / RSTRIDE>{});
      if constexpr (LOADS) {
        if constexpr (g == 1) set_m0_fn();
        if constexpr (g >= 3 && g <= 31 && (g - 3) % 4 == 0) loader(IC<(g - 3) / 4>{});
      }
    });
  };

  // Step kt at ring phase P.  KIND 2: a step that loads A(kt+2) (before its barrier, into B(kt-1)'s old slot) and
  // B(kt+2) (behind it, into A(kt)'s slot); KIND 1: the second to last step (nothing left to load); KIND 0: the
  // last step (no barrier, no next fragments).
  auto step = [&](TileState& t, int kt, auto phase_tag, auto kind_tag, auto nv_tag, auto sp_tag) __attribute__((always_inline)) {
    constexpr int P = decltype(phase_tag)::value, KIND = decltype(kind_tag)::value, NV = decltype(nv_tag)::value;
    using SA = IC<slot_of_a(P)>;
    using SB = IC<slot_of_b(P)>;
    using NA = IC<slot_of_a((P + 1) % NSLOT)>;
    using NB = IC<slot_of_b((P + 1) % NSLOT)>;
    constexpr int LA = slot_of_a((P + 2) % NSLOT);
    constexpr int NREADS = NV == 0 ? 0 : 2 * NV * A_OPS_PER_BLK + 8 * B_OPS_PER_BLK;
    if constexpr (KIND == 2 && GATHER_A) {
      // the tokens of A(kt+2) were fetched a step ago and are covered by that step's wait; those of A(kt+3)
      // are requested before the loads of A(kt+2), the only ones this step's wait leaves in flight
      apply_tok(t, t.tokn);
      if (kt + 3 < t.nk) fetch_tok(t, kt + 3, t.tokn);
    }
    sub_step(IC<0>{}, nv_tag, IC<NREADS>{},
             [&](auto op) __attribute__((always_inline)) { read_op(SA{}, SB{}, IC<1>{}, IC<1>{}, nv_tag, op); },
             IC<KIND == 2 ? 1 : 0>{},
             [&]() __attribute__((always_inline)) { set_m0<LA * TILE_BYTES>(lds_fill); },
             [&](auto i) __attribute__((always_inline)) { a_part(t, kt + 2, i, sp_tag); });
    if constexpr (KIND == 2) a_end(t, kt + 2);
    lds_wait<0>();
    if constexpr (KIND >= 1) {
      if constexpr (KIND == 2) wait_vm<8>(); else wait_vm<0>();   // this wave's loads of A(kt+2) may stay in flight
      wg_barrier();
    }
    if constexpr (KIND == 2 && GATHER_B) apply_tok(t, t.tokn);   // fetched a step ago, older than the loads of A(kt+2)
    sub_step(IC<1>{}, nv_tag, IC<KIND >= 1 ? NREADS : 0>{},
             [&](auto op) __attribute__((always_inline)) { read_op(NA{}, NB{}, IC<0>{}, IC<0>{}, nv_tag, op); },
             IC<KIND == 2 ? 1 : 0>{},
             [&]() __attribute__((always_inline)) { set_m0<SA::value * TILE_BYTES>(lds_fill); },
             [&](auto i) __attribute__((always_inline)) { b_part(t, kt + 2, i, sp_tag); });
    if constexpr (KIND == 2) {
      b_end(t, kt + 2);
      if constexpr (GATHER_B) {
        // a whole step ahead of their use; the next step's wait covers them (they are older than its A loads)
        if (kt + 3 < t.nk) fetch_tok(t, kt + 3, t.tokn);
      }
    }
    lds_wait<0>();
  };

  // The first loads of a tile: steps 0 and 1 into the slots of phases p0 and p0 + 1; awaited when the tile's
  // main loop starts.  (Requesting them before the epilogue of the tile before, with the epilogue staged in the
  // one slot they leave free, was built and measured: the loads' latency disappears, 3.5 us per tile, and the
  // step takes as long as before, because the chip is power-limited and the main loops slow down by what the
  // idle phases no longer give back.)
  auto first_loads = [&](TileState& t) __attribute__((always_inline)) {
    if (t.nk <= 0) return;
    const int p0 = t.p0;
    const int p1 = (p0 + 1) % NSLOT;
    const uint32_t m_a0 = lds_fill + ((2 * p0) % NSLOT) * TILE_BYTES, m_b0 = lds_fill + ((2 * p0 + 1) % NSLOT) * TILE_BYTES;
    const uint32_t m_a1 = lds_fill + ((2 * p1) % NSLOT) * TILE_BYTES, m_b1 = lds_fill + ((2 * p1 + 1) % NSLOT) * TILE_BYTES;
    auto a_unit = [&](int kt, uint32_t m) __attribute__((always_inline)) {
      set_m0_rt(m);
      asm volatile("s_nop 0" ::: "memory");
      static_for<8>([&](auto i) { a_part(t, kt, i, IC<2>{}); });
      a_end(t, kt);
    };
    auto b_unit = [&](int kt, uint32_t m) __attribute__((always_inline)) {
      set_m0_rt(m);
      asm volatile("s_nop 0" ::: "memory");
      static_for<8>([&](auto i) { b_part(t, kt, i, IC<2>{}); });
      b_end(t, kt);
    };
    if constexpr (GATHER_B) {
      // the tokens of steps 0 and 1 are requested first and are older than the loads of A(0), A(1): one wait for both
      fetch_tok(t, 0, t.tokn);
      if (t.nk > 1) fetch_tok(t, 1, t.tokn1);
      a_unit(0, m_a0);
      if (t.nk > 1) { a_unit(1, m_a1); wait_vm<16>(); } else { wait_vm<8>(); }
      apply_tok(t, t.tokn);
      b_unit(0, m_b0);
      if (t.nk > 1) { apply_tok(t, t.tokn1); b_unit(1, m_b1); }
    } else if constexpr (GATHER_A) {
      fetch_tok(t, 0, t.tokn);
      if (t.nk > 1) fetch_tok(t, 1, t.tokn1);
      b_unit(0, m_b0);
      if (t.nk > 1) { b_unit(1, m_b1); wait_vm<16>(); } else { wait_vm<8>(); }
      apply_tok(t, t.tokn);
      a_unit(0, m_a0);
      if (t.nk > 1) {
        apply_tok(t, t.tokn1);
        if (t.nk > 2) fetch_tok(t, 2, t.tokn);   // applied at the start of step 0: older than the loads of A(1)
        a_unit(1, m_a1);
      }
    } else {
      b_unit(0, m_b0);
      a_unit(0, m_a0);
      if (t.nk > 1) { b_unit(1, m_b1); a_unit(1, m_a1); }
    }
    if constexpr (GATHER_B) {
      if (t.nk > 2) fetch_tok(t, 2, t.tokn);   // applied behind step 0's barrier, whose wait covers it
    }
  };
  auto main_loop = [&](TileState& t, auto nv_tag) __attribute__((always_inline)) {
    if (t.nk <= 0) return;
    const int p0 = t.p0, nmain = t.nmain;
    // The tile's first loads are awaited; those of step 1 may stay in flight (the stores of the epilogue before
    // are older than all of them, and loads complete in order among themselves).
    if (GATHER_A || GATHER_B || t.nk <= 1) wait_vm<0>(); else wait_vm<16>();
    wg_barrier();
    // ---- first fragments: sub-step 0 of step 0, from the slots of phase p0
    constexpr int NV = decltype(nv_tag)::value;
    constexpr int NREADS = NV == 0 ? 0 : 2 * NV * A_OPS_PER_BLK + 8 * B_OPS_PER_BLK;
    auto first_reads = [&](auto phase_tag) __attribute__((always_inline)) {
      constexpr int P = decltype(phase_tag)::value;
      static_for<NREADS>([&](auto op) { read_op(IC<slot_of_a(P)>{}, IC<slot_of_b(P)>{}, IC<0>{}, IC<0>{}, nv_tag, op); });
    };
    switch (p0) {
      case 0: first_reads(IC<0>{}); break;
      case 1: first_reads(IC<1>{}); break;
      case 2: first_reads(IC<2>{}); break;
      case 3: first_reads(IC<3>{}); break;
      default: first_reads(IC<4>{}); break;
    }
    lds_wait<0>();
    asm volatile("s_nop 7" ::: "memory");   // the accumulators were cleared by vector-ALU writes: keep the first MFMA clear of them
    // ---- the steps that load, in rounds of the five phases (the first round starts at p0)
    int kt = 0;
    int skip = p0;
    while (kt < nmain) {
      if (skip <= 0) { step(t, kt, IC<0>{}, IC<2>{}, nv_tag, IC<0>{}); ++kt; }
      if (skip <= 1) { step(t, kt, IC<1>{}, IC<2>{}, nv_tag, IC<0>{}); ++kt; }
      if (skip <= 2) { step(t, kt, IC<2>{}, IC<2>{}, nv_tag, IC<0>{}); ++kt; }
      if (skip <= 3) { step(t, kt, IC<3>{}, IC<2>{}, nv_tag, IC<0>{}); ++kt; }
      step(t, kt, IC<4>{}, IC<2>{}, nv_tag, IC<0>{}); ++kt;
      skip = 0;
    }
    // ---- the last three steps
    if (t.nk >= 3) step(t, t.nk - 3, IC<0>{}, IC<2>{}, nv_tag, IC<is_wgrad(MODE) ? 1 : 0>{});
    if (t.nk >= 2) step(t, t.nk - 2, IC<1>{}, IC<1>{}, nv_tag, IC<0>{});
    step(t, t.nk - 1, IC<2>{}, IC<0>{}, nv_tag, IC<0>{});
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMAs have written before the accumulators are read
  };
  // one copy of the loop per number of live 32-row groups: a wave whose 128 rows all lie past the
  // expert's end only keeps the loads and barriers going
  auto run_main = [&](TileState& t) __attribute__((always_inline)) {
    if constexpr (is_wgrad(MODE)) {
      main_loop(t, IC<4>{});
    } else {
      switch (t.nv) {
        case 4: main_loop(t, IC<4>{}); break;
        case 3: main_loop(t, IC<3>{}); break;
        case 2: main_loop(t, IC<2>{}); break;
        case 1: main_loop(t, IC<1>{}); break;
        default: main_loop(t, IC<0>{}); break;
      }
    }
  };
  // ---------------- epilogue -----------------------------------------------------
  // acc[i][j][c] is the wave's element (row, col) with row = 16 i + (lane & 15) and col = 16 j + 4 (lane / 16) + c.
  // The wave stages bf16 rows of 256 bytes in 8 KB of LDS of its own (its share of ring slot 0; 16-byte pieces
  // swizzled by the row), a few rows at a time, and stores 16 bytes per lane in full row segments.
  // The accumulators are read out of the accumulation registers at the point of use, by hand: left to the
  // compiler they are moved (and spilled) in bulk where the copies of the main loop join.
  auto accq = [&](auto i_tag, auto j_tag) __attribute__((always_inline)) -> f32x4_t {
    constexpr int i = decltype(i_tag)::value, j = decltype(j_tag)::value;
    f32x4_t v;
    float x;
    const float c0 = acc[i][j][0], c1 = acc[i][j][1], c2 = acc[i][j][2], c3 = acc[i][j][3];
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(c0));  v[0] = x;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(c1));  v[1] = x;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(c2));  v[2] = x;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(c3));  v[3] = x;
    return v;
  };
  // GATE_UP with gate weights folded into h, DGRAD_H_GATE: the weights of the lane's eight rows, requested by
  // hand right behind the main loop and awaited by hand where the epilogue first needs them.
  float wv[8];
  auto fetch_row_weights = [&](const TileState& t, const float* rw) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int r = t.m0 + wm * 128 + i * 16 + (lane & 15);  if (r > t.m_end - 1) r = t.m_end - 1;
      const float* ptr = rw + r;
      asm volatile("global_load_dword %0, %1, off" : "=v"(wv[i]) : "v"(ptr) : "memory");
    }
  };

  auto epilogue = [&](const TileState& t) __attribute__((always_inline)) {
    const ArgPtr ae = reload_args<ARG>();     // the epilogue reads its arguments afresh
    int tid = tid0;                           // laundered as in setup_tile
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
    const int m0 = t.m0, m_end = t.m_end, n0 = t.n0;
    const int grow0 = m0 + wm * 128;                                     // wave's first output row
    const int gcol0 = n0 + wn * (MODE == GATE_UP ? 64 : 128);            // wave's first output column
    char* stage = lds + wave * 8192;
    // address of the 8 bytes of columns 4 lq .. + 3 of 16-column block `blk` in staged row `row`
    auto quad_addr = [&](int row, int blk) __attribute__((always_inline)) -> char* {
      return stage + row * 256 + (((2 * blk + (lq >> 1)) ^ (row & 15)) << 4) + (lq & 1) * 8;
    };
    auto put_quad = [&](int row, int blk, const f32x4_t& v) __attribute__((always_inline)) {
      u32x2 o;
      o.x = pack_bf16(v[0], v[1]);
      o.y = pack_bf16(v[2], v[3]);
      *reinterpret_cast<u32x2*>(quad_addr(row, blk)) = o;
    };
    // Stores ROWS staged rows of RB bytes (pieces swizzled by row & (RB / 16 - 1); region at `base`) to out rows
    // first_row .. (row stride ld): each row's PIECES 16-byte pieces from piece PIECE0 on go to columns
    // col0 + 8 piece.  The LDS reads of up to eight passes are issued together, then their stores (one wave per
    // SIMD: nothing else would cover the latency of a read-then-store chain).  When every row and column of the
    // block exists (a wave-uniform test) the stores are unconditional and their addresses one add apart;
    // otherwise each is masked by its row and column.  NT: the output is not read again soon (g and u: not before
    // the backward pass; dWg and dWu: not by this layer at all), so its stores are marked non-temporal and leave the
    // caches to what the next kernels read (measured: 0.4-0.6 % of the step, most of it in the kernels that follow).
    auto flush = [&](auto nt_tag, const char* base, auto rb_tag, uint16_t* out, size_t ld, int first_row, auto rows_tag, auto piece0_tag,
                     auto pieces_tag, int col0, int ncols) __attribute__((always_inline)) {
      constexpr int RB = decltype(rb_tag)::value, ROWS = decltype(rows_tag)::value;
      constexpr bool NT = decltype(nt_tag)::value != 0;
      typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
      auto put = [&](char* p, const u32x4& v) __attribute__((always_inline)) {
        if constexpr (NT) { u32x4_nt w = {v.x, v.y, v.z, v.w}; __builtin_nontemporal_store(w, reinterpret_cast<u32x4_nt*>(p)); }
        else *reinterpret_cast<u32x4*>(p) = v;
      };
      constexpr int PIECE0 = decltype(piece0_tag)::value, PIECES = decltype(pieces_tag)::value;
      constexpr int RPP = 64 / PIECES, PASSES = ROWS / RPP, SWZ = RB / 16 - 1;
      const int prow = lane / PIECES, piece = lane % PIECES;
      const int gc = col0 + piece * 8;
      const bool whole = first_row + ROWS <= m_end && col0 + PIECES * 8 <= ncols;
      char* const p0 = reinterpret_cast<char*>(out + static_cast<size_t>(first_row + prow) * ld + gc);
      const size_t pass_bytes = static_cast<size_t>(RPP) * ld * 2;
      static_for<(PASSES + 7) / 8>([&](auto b_tag) {
        constexpr int P0 = decltype(b_tag)::value * 8;
        constexpr int NB = PASSES - P0 < 8 ? PASSES - P0 : 8;
        u32x4 v[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
          const int row = (P0 + k) * RPP + prow;
          v[k] = *reinterpret_cast<const u32x4*>(base + row * RB + (((PIECE0 + piece) ^ (row & SWZ)) << 4));
        }
        if (whole) {
#pragma unroll
          for (int k = 0; k < NB; ++k) put(p0 + (P0 + k) * pass_bytes, v[k]);
        } else {
#pragma unroll
          for (int k = 0; k < NB; ++k) {
            const int gr = first_row + (P0 + k) * RPP + prow;
            if (gr < m_end && gc < ncols) put(p0 + (P0 + k) * pass_bytes, v[k]);
          }
        }
      });
    };

    if constexpr (MODE == GATE_UP) {
      // blocks 0-3 are g, blocks 4-7 the same columns of u.  Eight parts of 16 rows: g in pieces 0-7 and u in
      // pieces 8-15 of 256-byte rows, h = silu(g) * u (from the fp32 accumulators, times the row's gate weight if
      // the caller folds the weights into h) in 128-byte rows behind them.
      const bool weighted = ae->row_weight != nullptr;
      if (weighted) {
        wait_vm<0>();
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(wv[i]));
      }
      char* hstage = stage + 16 * 256;
      static_for<8>([&](auto i_tag) {
        constexpr int i = decltype(i_tag)::value;
        const int row = l16;
        const float w = weighted ? wv[i] : 1.f;
        static_for<4>([&](auto j_tag) {
          constexpr int j = decltype(j_tag)::value;
          const f32x4_t gv = accq(i_tag, IC<j>{});
          const f32x4_t uv = accq(i_tag, IC<j + 4>{});
          put_quad(row, j, gv);
          put_quad(row, j + 4, uv);
          u32x2 o;
          float h[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) h[c] = silu_f(gv[c]) * uv[c] * w;
          o.x = pack_bf16(h[0], h[1]);
          o.y = pack_bf16(h[2], h[3]);
          *reinterpret_cast<u32x2*>(hstage + row * 128 + (((2 * j + (lq >> 1)) ^ (row & 7)) << 4) + (lq & 1) * 8) = o;
        });
        __builtin_amdgcn_wave_barrier();
        flush(IC<1>{}, stage, IC<256>{}, ae->O0, ae->N, grow0 + i * 16, IC<16>{}, IC<0>{}, IC<8>{}, gcol0, ae->N);
        flush(IC<1>{}, stage, IC<256>{}, ae->O1, ae->N, grow0 + i * 16, IC<16>{}, IC<8>{}, IC<8>{}, gcol0, ae->N);
        flush(IC<0>{}, hstage, IC<128>{}, ae->O2, ae->N, grow0 + i * 16, IC<16>{}, IC<0>{}, IC<8>{}, gcol0, ae->N);
        __builtin_amdgcn_wave_barrier();
      });
    } else if constexpr (is_dgrad_h(MODE)) {
      // In eight parts of 16 rows, staged alternately in the wave's share of the first and of the second ring
      // slot: g rows at [0, 4K), u rows at [4K, 8K) of the part's buffer, overwritten in place by dg and du.
      // Order of the memory operations of part p: compute p; await the g/u rows of part p+1 and stage them;
      // store part p; request the g/u rows of part p+2.  Waiting for loads also waits for every store issued
      // before them (stores and loads share a counter and complete in no fixed order), so the wait is placed
      // where the youngest stores are a whole part old, never right behind a part's own stores.
      // DGRAD_H_GATE: the accumulators hold dh0 = dout[token] . Wd; the row's gate weight w turns them into
      // dh = w dh0, and the sum over a 64-column strip of dh0 * silu(g) * u is the strip's share of the
      // gradient of w (a lane holds 16 of the strip's columns of its row, lanes ^ 16, ^ 32 the others).
      constexpr bool GATE = (MODE == DGRAD_H_GATE);
      constexpr int GU_PASSES = 4;   // 16 rows x 16 pieces = 256 pieces of 16 bytes, 64 per pass
      constexpr int UOFF = 4096;
      u32x4 pg[GU_PASSES], pu[GU_PASSES];
      auto gu_load = [&](int part) __attribute__((always_inline)) {
        const int ncol = ae->N;
        const uint16_t* gsrc = ae->G;
        const uint16_t* usrc = ae->U;
        const int r0 = grow0 + part * 16;
        if (r0 + 16 <= m_end && gcol0 + 128 <= ncol) {   // wave-uniform: the whole part exists, nothing to clamp
          const size_t o = static_cast<size_t>(r0 + (lane >> 4)) * ncol + gcol0 + (lane & 15) * 8;
          const size_t pass = static_cast<size_t>(4) * ncol;
#pragma unroll
          for (int p = 0; p < GU_PASSES; ++p) {
            pg[p] = *reinterpret_cast<const u32x4*>(gsrc + o + p * pass);
            pu[p] = *reinterpret_cast<const u32x4*>(usrc + o + p * pass);
          }
          return;
        }
#pragma unroll
        for (int p = 0; p < GU_PASSES; ++p) {
          const int row = p * 4 + (lane >> 4), piece = lane & 15;
          int gr = r0 + row;  if (gr > m_end - 1) gr = m_end - 1;
          int gc = gcol0 + piece * 8;  if (gc > ncol - 8) gc = ncol - 8;
          const size_t o = static_cast<size_t>(gr) * ncol + gc;
          pg[p] = *reinterpret_cast<const u32x4*>(gsrc + o);
          pu[p] = *reinterpret_cast<const u32x4*>(usrc + o);
        }
      };
      auto gu_stage = [&](char* buf) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < GU_PASSES; ++p) {
          const int row = p * 4 + (lane >> 4), piece = lane & 15;
          const int so = row * 256 + ((piece ^ (row & 15)) << 4);
          *reinterpret_cast<u32x4*>(buf + so) = pg[p];
          *reinterpret_cast<u32x4*>(buf + UOFF + so) = pu[p];
        }
      };
      char* const bufs[2] = {stage, stage + TILE_BYTES};
      int qoff[8];                  // offsets of the lane's quads in a part's buffer: the same for every part
#pragma unroll
      for (int j = 0; j < 8; ++j) qoff[j] = static_cast<int>(quad_addr(l16, j) - stage);
      if constexpr (GATE) {
        wait_vm<0>();               // the row weights requested behind the main loop
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(wv[i]));
      }
      gu_load(0);
      gu_stage(bufs[0]);
      gu_load(1);
      float dpart[8][2];
      static_for<8>([&](auto part_tag) {
        constexpr int part = decltype(part_tag)::value;
        const int first = grow0 + part * 16;
        char* const buf = bufs[part & 1];
        const float wrow = GATE ? wv[part] : 1.f;
        float dsum[2] = {0.f, 0.f};
        __builtin_amdgcn_wave_barrier();
        // the lane's eight g and u quads of the part, read in one go: the quads are overwritten in place below, so
        // reads issued one by one would each wait behind the previous quad's write
        u32x2 gqs[8], uqs[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          gqs[j] = *reinterpret_cast<const u32x2*>(buf + qoff[j]);
          uqs[j] = *reinterpret_cast<const u32x2*>(buf + qoff[j] + UOFF);
        }
        static_for<8>([&](auto j_tag) {
          constexpr int j = decltype(j_tag)::value;
          const f32x4_t dhv = accq(part_tag, j_tag);
          char* ga = buf + qoff[j];
          char* ua = ga + UOFF;
          const u32x2 gq = gqs[j];
          const u32x2 uq = uqs[j];
          const float g4[4] = {bf16lo(gq.x), bf16hi(gq.x), bf16lo(gq.y), bf16hi(gq.y)};
          const float u4[4] = {bf16lo(uq.x), bf16hi(uq.x), bf16lo(uq.y), bf16hi(uq.y)};
          float dg[4], du[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const float sg = sigmoid_f(g4[c]);
            if constexpr (GATE) {
              const float dh0 = dhv[c];
              const float sl = g4[c] * sg;                 // silu(g)
              const float t0 = dh0 * u4[c];
              dsum[j >> 2] = __builtin_fmaf(t0, sl, dsum[j >> 2]);
              du[c] = (dh0 * wrow) * sl;
              dg[c] = (t0 * wrow) * (sg * __builtin_fmaf(g4[c], 1.0f - sg, 1.0f));
            } else {
              const float dh = dhv[c];
              const float x = dh * sg;                     // shared by both derivatives
              du[c] = x * g4[c];
              dg[c] = (x * u4[c]) * __builtin_fmaf(g4[c], 1.0f - sg, 1.0f);
            }
          }
          u32x2 o;
          o.x = pack_bf16(dg[0], dg[1]);  o.y = pack_bf16(dg[2], dg[3]);
          *reinterpret_cast<u32x2*>(ga) = o;
          o.x = pack_bf16(du[0], du[1]);  o.y = pack_bf16(du[2], du[3]);
          *reinterpret_cast<u32x2*>(ua) = o;
        });
        if constexpr (GATE) {
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            float x = dsum[s2];
            x += __shfl_xor(x, 16, 64);
            x += __shfl_xor(x, 32, 64);
            dpart[part][s2] = x;
          }
        }
        __builtin_amdgcn_wave_barrier();
        if constexpr (part + 1 < 8) gu_stage(bufs[(part + 1) & 1]);   // awaits the loads of part + 1
        __builtin_amdgcn_wave_barrier();
        flush(IC<0>{}, buf, IC<256>{}, ae->O0, ae->N, first, IC<16>{}, IC<0>{}, IC<16>{}, gcol0, ae->N);
        flush(IC<0>{}, buf + UOFF, IC<256>{}, ae->O1, ae->N, first, IC<16>{}, IC<0>{}, IC<16>{}, gcol0, ae->N);
        __builtin_amdgcn_wave_barrier();
        if constexpr (part + 2 < 8) gu_load(part + 2);
      });
      if constexpr (GATE) {
        // the strips' shares of the gate gradient, stored behind everything else (a store in the middle of a
        // part would be one more thing the next wait for loads has to sit out)
        const int strips = ae->N >> 6;
        static_for<8>([&](auto part_tag) {
          constexpr int part = decltype(part_tag)::value;
          const int r = grow0 + part * 16 + l16;
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            if (gcol0 + s2 * 64 < ae->N) {     // a strip past the last column holds repeated columns: no share
              float* part_out = ae->dgate_part + ((gcol0 >> 6) + s2);
              if (lq == 0 && r < m_end) part_out[static_cast<size_t>(r) * strips] = dpart[part][s2];
            }
          }
        });
      }
    } else {
      uint16_t* out = t.second ? ae->O1 : ae->O0;
      if constexpr (is_wgrad(MODE)) out += static_cast<size_t>(t.e) * ae->M * ae->N;
      // four parts of 32 rows
      static_for<4>([&](auto part_tag) {
        constexpr int part = decltype(part_tag)::value;
        static_for<2>([&](auto i2_tag) {
          constexpr int i2 = decltype(i2_tag)::value;
          static_for<8>([&](auto j_tag) { put_quad(i2 * 16 + l16, decltype(j_tag)::value, accq(IC<part * 2 + i2>{}, j_tag)); });
        });
        __builtin_amdgcn_wave_barrier();
        flush(IC<(MODE == WGRAD_GATHER) ? 1 : 0>{}, stage, IC<256>{}, out, ae->N, grow0 + part * 32, IC<32>{}, IC<0>{}, IC<16>{}, gcol0, ae->N);
        __builtin_amdgcn_wave_barrier();
      });
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wave's staging reads are done
  };

  // ---------------- the tile loop ------------------------------------------------
  int tile = first_tile;
  if (tile < total) {
    TileState cur;
    setup_tile(tile, cur);
    first_loads(cur);
    for (;;) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
      run_main(cur);
      wg_barrier();                             // every wave is done with the operand tiles
      if constexpr (MODE == GATE_UP) {
        if (a.row_weight != nullptr) fetch_row_weights(cur, a.row_weight);
      }
      if constexpr (MODE == DGRAD_H_GATE) fetch_row_weights(cur, a.row_weight);
      epilogue(cur);
      // a wave stages in, and loads into, its own 8 KB of a slot only: no barrier between epilogue and loads
      tile += gridDim.x;
      if (tile >= total) break;
      setup_tile(tile, cur);
      first_loads(cur);
    }
  }
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

// Per-device facts, looked up once per device: HIP keeps function attributes and the number of compute
// units per device, and a process may drive several.  Races between host threads are benign (both write
// the same values).
constexpr int MAX_DEVICES = 64;
int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = 0; }
  return dev >= 0 && dev < MAX_DEVICES ? dev : 0;
}
// Workgroups of the persistent launch: one per compute unit (the 160 KB of LDS allow no more),
// a multiple of 8 so that every XCD gets the same share, and no more than there can be tiles.
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

// byte offsets of gathered rows are 32-bit lane offsets from the start of x (T*width*2 bytes just under 4 GiB at most)
bool bad_gather(const moe_bf16* x, int T, const int32_t* row_token, int width) {
  return !x || !row_token || T <= 0 || !moe_aligned16(row_token) ||
         static_cast<unsigned long long>(T) * width * sizeof(moe_bf16) > 0xFFFFFFFFull - 65536;   // lane offsets carry a small bias on top
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
  // dxp = dg . Wg + du . Wu ; dWg = dg^T xp and dWu = du^T xp (one list: both read the same rows of xp)
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
  // dgrad_x first: its tiles are the long ones, the weight gradients' many short tiles fill its tail
  if (row_token != nullptr) return launch_gemm_pair<DGRAD_X, WGRAD_GATHER>(b, w, tiles, s, "gemm_wgrad_gate_up+dgrad_x");
  return launch_gemm_pair<DGRAD_X, WGRAD>(b, w, tiles, s, "gemm_wgrad_gate_up+dgrad_x");
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
  // dgrad_x first: its tiles are the long ones, the weight gradients' many short tiles fill its tail.  (The other
  // order used to pay off through dxp still lying in the last-level cache when moe_permute_bwd read it; since that
  // kernel streams its rows with non-temporal loads it no longer depends on that.)
  return launch_gemm_pair<DGRAD_X, WGRAD_GATHER>(b, w, 2ll * w.n_tiles * w.m_tiles_cap * E + static_cast<long long>(b.n_tiles) * m_tiles,
                                                 s, "gemm_wgrad_gate_up+dgrad_x");
}
