// Stages 2-3 of Algorithm 1 (token counting, index generation) and the Stage-4
// gather, as an atomics-free stable counting sort:
//
//   count   the (token, slot) pairs are cut into at most 256 chunks of consecutive pairs; one
//           workgroup per chunk counts its pairs per local expert: each wave finds, with one
//           ballot per bit of the expert id, the lanes of a 64-pair batch that chose the same
//           expert, and the lowest lane of each such group adds the group size to the wave's own
//           LDS row: no atomic anywhere.  -> hist[chunk][expert].  When the routing runs in the
//           same call, the routing kernel counts its own winners and this launch does not exist.
//   place   every workgroup first sums the table's columns: over all chunks (the experts' totals,
//           whose exclusive scan is expert_offsets) and over the chunks in front of its own (the
//           first row of its (expert, chunk) cell).  This is the paper's cum_token_counts /
//           partial_cum_token_counts at chunk granularity, recomputed by every workgroup from a
//           table that stays in L2 instead of by a kernel of its own.  It then recounts its pairs,
//           derives each wave's first row per expert, and ranks pairs inside a batch by the
//           popcount of the lower lanes that chose the same expert -> slot_row, row_token.
//   rows    one wave per token copies x[t] to its (up to k) grouped rows with
//           16-byte accesses: x is read once, xp is written in full rows.
#include "perm_common.h"

namespace {

__global__ __launch_bounds__(PERM_THREADS) void permute_count_kernel(const int32_t* __restrict__ topk_idx, int n,
                                                                     int e_begin, int e_count, int nbits, int chunk,
                                                                     int32_t* __restrict__ hist) {
  __shared__ int wcnt[PERM_WAVES][MOE_MAX_EXPERTS];
  const int tid = threadIdx.x, w = tid / MOE_WAVE;
  for (int e = tid; e < e_count; e += PERM_THREADS) {
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) wcnt[v][e] = 0;
  }
  __syncthreads();
  const int first = blockIdx.x * chunk;
  const int len = min(chunk, n - first);
  count_wave_span(len, nbits, wcnt[w], [&](int i) {
    const int e = topk_idx[first + i] - e_begin;
    return (e < 0 || e >= e_count) ? -1 : e;
  });
  __syncthreads();
  for (int e = tid; e < e_count; e += PERM_THREADS) {
    int s = 0;
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) s += wcnt[v][e];
    hist[static_cast<size_t>(blockIdx.x) * e_count + e] = s;
  }
}

__global__ __launch_bounds__(PERM_THREADS) void permute_place_kernel(const int32_t* __restrict__ topk_idx, int n, int k,
                                                                     int e_begin, int e_count, int nbits, int chunk,
                                                                     const int32_t* __restrict__ hist,
                                                                     int32_t* __restrict__ expert_offsets,
                                                                     int32_t* __restrict__ row_token,
                                                                     int32_t* __restrict__ slot_row,
                                                                     const float* __restrict__ topk_w,
                                                                     float* __restrict__ row_weight) {
  __shared__ int wcnt[PERM_WAVES][MOE_MAX_EXPERTS];
  // partial column sums, [part][expert]: parts * e_count <= 1024 entries (before: rows of the chunks in front
  // of this one; total: the expert's rows)
  __shared__ __attribute__((aligned(16))) int part_before[2 * MOE_MAX_EXPERTS];
  __shared__ __attribute__((aligned(16))) int part_total[2 * MOE_MAX_EXPERTS];
  __shared__ int first_row[MOE_MAX_EXPERTS];                  // first row of this chunk's cell of the expert
  const int tid = threadIdx.x, w = tid / MOE_WAVE, lane = tid % MOE_WAVE;
  const int b = blockIdx.x, nblocks = gridDim.x;

  // this chunk's pairs; the lane's pair of its wave's first batch is loaded now, ahead of the table
  const int first = b * chunk;
  const int len = min(chunk, n - first);
  auto load_local = [&](int i) {
    const int e = topk_idx[first + i] - e_begin;
    return (e < 0 || e >= e_count) ? -1 : e;
  };
  const int span = perm_wave_span(len);
  const int lo = w * span, hi = min(len, lo + span);
  const int i_pre = lo + lane;
  const int e_pre = i_pre < hi ? load_local(i_pre) : -1;
  auto local = [&](int i) { return i == i_pre ? e_pre : load_local(i); };

  // ---- column sums of the table: a thread owns `vec` neighbouring columns of every parts-th chunk ----
  const int vec = (e_count % 4 == 0) ? 4 : 1;                  // 16-byte reads when the rows allow it
  const int ncol = e_count / vec;                             // column groups
  int cols = 1;
  while (cols < ncol && cols < PERM_THREADS) cols <<= 1;
  const int parts = PERM_THREADS / cols;                      // parts * e_count <= 256 / cols * 4 * cols = 1024
  const int p = tid / cols;
  for (int cg = tid % cols; cg < ncol; cg += (parts == 1 ? PERM_THREADS : (1 << 30))) {
    int bef[4] = {0, 0, 0, 0}, tot[4] = {0, 0, 0, 0};
    if (vec == 4) {
#pragma unroll 16
      for (int q = p; q < nblocks; q += parts) {
        const int4 v = *reinterpret_cast<const int4*>(hist + static_cast<size_t>(q) * e_count + cg * 4);
        const int m = q < b ? -1 : 0;
        tot[0] += v.x; tot[1] += v.y; tot[2] += v.z; tot[3] += v.w;
        bef[0] += v.x & m; bef[1] += v.y & m; bef[2] += v.z & m; bef[3] += v.w & m;
      }
    } else {
#pragma unroll 8
      for (int q = p; q < nblocks; q += parts) {
        const int v = hist[static_cast<size_t>(q) * e_count + cg];
        tot[0] += v;
        bef[0] += q < b ? v : 0;
      }
    }
    for (int j = 0; j < vec; ++j) {
      part_before[p * e_count + cg * vec + j] = bef[j];
      part_total[p * e_count + cg * vec + j] = tot[j];
    }
  }
  for (int e = tid; e < e_count; e += PERM_THREADS) {
#pragma unroll
    for (int v = 0; v < PERM_WAVES; ++v) wcnt[v][e] = 0;
  }
  __syncthreads();
  // ---- the first wave adds up the parts (ceil(e_count / 64) experts per lane), scans the experts' totals and
  //      leaves in first_row the first row of this chunk's cell of every expert ----
  if (w == 0) {
    const int seg = (e_count + MOE_WAVE - 1) / MOE_WAVE;   // <= MOE_MAX_EXPERTS / 64 = 8
    int befs[MOE_MAX_EXPERTS / MOE_WAVE], tots[MOE_MAX_EXPERTS / MOE_WAVE];
    int s = 0;
#pragma unroll
    for (int j = 0; j < MOE_MAX_EXPERTS / MOE_WAVE; ++j) {
      const int e = lane * seg + j;
      int bef = 0, tot = 0;
      if (j < seg && e < e_count) {
        for (int q = 0; q < parts; ++q) { bef += part_before[q * e_count + e]; tot += part_total[q * e_count + e]; }
      }
      befs[j] = bef;
      tots[j] = tot;
      s += tot;
    }
    int inc = s;
#pragma unroll
    for (int d = 1; d < MOE_WAVE; d <<= 1) {
      const int o = __shfl_up(inc, d, MOE_WAVE);
      if (lane >= d) inc += o;
    }
    int run = inc - s;
#pragma unroll
    for (int j = 0; j < MOE_MAX_EXPERTS / MOE_WAVE; ++j) {
      const int e = lane * seg + j;
      if (j < seg && e < e_count) {
        first_row[e] = run + befs[j];
        if (b == 0) expert_offsets[e] = run;
        run += tots[j];
      }
    }
    if (b == 0 && lane == MOE_WAVE - 1) expert_offsets[e_count] = inc;
  }

  // ---- this chunk: counts per wave, each wave's first row per expert, ranks ----
  count_wave_span(len, nbits, wcnt[w], local);
  __syncthreads();
  for (int e = tid; e < e_count; e += PERM_THREADS) {
    int base = first_row[e];
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
  for (int f0 = lo; f0 < hi; f0 += MOE_WAVE) {
    const int i = f0 + lane;
    const int e = i < hi ? local(i) : -1;
    int row = -1;
    const uint64_t m = same_expert_mask(e, nbits);
    if (m != 0) {
      const int base = next[e];                      // every lane of the group reads the same counter
      row = base + __builtin_popcountll(m & lt);
      __builtin_amdgcn_wave_barrier();
      if (lane == __builtin_ctzll(m)) next[e] = base + __builtin_popcountll(m);
    }
    __builtin_amdgcn_wave_barrier();
    if (i < hi) {
      const int idx = first + i;
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

// Chunks of the plain path (topk_idx given): whole multiples of 256 pairs, as few as keep the table at
// perm_max_chunks rows.
inline int perm_chunk_pairs(long long n, int e_count) {
  const long long units = (n + 255) / 256;
  const long long per = (units + perm_max_chunks(e_count) - 1) / perm_max_chunks(e_count);
  return static_cast<int>(per * 256);
}

}  // namespace

extern "C" size_t moe_permute_workspace_bytes(int T, int k, int e_count) {
  if (T <= 0 || k <= 0 || e_count <= 0) return 0;
  // one table row per 256 pairs covers every chunking (chunks never hold fewer pairs than that)
  const size_t rows = (static_cast<size_t>(T) * k + 255) / 256;
  return (rows * e_count * sizeof(int32_t) + 16 + 255) & ~static_cast<size_t>(255);
}

namespace {
void launch_rows(const moe_bf16* x, const int32_t* slot_row, int T, int d, int k, moe_bf16* xp, hipStream_t s) {
  const int chunks = d / 8;
  dim3 grid((T + 3) / 4), block(256);
  const uint4* xs = reinterpret_cast<const uint4*>(x);
  uint4* xd = reinterpret_cast<uint4*>(xp);
  if (chunks <= 64)
    MOE_LAUNCH("permute_rows", permute_rows_kernel<1>, grid, block, 0, s, xs, slot_row, T, k, chunks, xd);
  else if (chunks <= 128)
    MOE_LAUNCH("permute_rows", permute_rows_kernel<2>, grid, block, 0, s, xs, slot_row, T, k, chunks, xd);
  else
    MOE_LAUNCH("permute_rows", permute_rows_kernel<4>, grid, block, 0, s, xs, slot_row, T, k, chunks, xd);
}

int check_permute_args(const moe_bf16* x, const int32_t* topk_idx, int T, int d, int E_total, int k, int e_begin,
                       int e_count, const int32_t* expert_offsets, const int32_t* row_token, const int32_t* slot_row,
                       const moe_bf16* xp, const void* ws, size_t ws_bytes) {
  // xp == NULL: index generation only (for callers that let the GEMMs gather the rows); x is not read then
  if (!topk_idx || !expert_offsets || !row_token || !slot_row || !ws || (xp && !x)) return MOE_ERR_INVALID;
  if (T <= 0 || d <= 0 || d % 8 != 0 || E_total <= 0 || k <= 0 || k > E_total) return MOE_ERR_INVALID;
  if (e_begin < 0 || e_count <= 0 || e_begin + e_count > E_total || e_count > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (static_cast<long long>(T) * k > 0x7FFFFFFFll / 2) return MOE_ERR_INVALID;
  if ((xp && (!moe_aligned16(x) || !moe_aligned16(xp))) || !moe_aligned16(ws) || !moe_aligned16(topk_idx) ||
      !moe_aligned16(slot_row) || !moe_aligned16(row_token) || !moe_aligned16(expert_offsets))
    return MOE_ERR_INVALID;
  if (ws_bytes < moe_permute_workspace_bytes(T, k, e_count)) return MOE_ERR_WORKSPACE;
  return MOE_OK;
}

int expert_bits(int e_count) {
  int nbits = 0;
  while ((1 << nbits) < e_count) ++nbits;
  return nbits;
}

int permute_impl(const moe_bf16* x, const int32_t* topk_idx, const float* topk_w, int T, int d, int E_total, int k,
                 int e_begin, int e_count, int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row,
                 float* row_weight, moe_bf16* xp, void* ws, size_t ws_bytes, void* stream) {
  const int bad = check_permute_args(x, topk_idx, T, d, E_total, k, e_begin, e_count, expert_offsets, row_token, slot_row,
                                     xp, ws, ws_bytes);
  if (bad != MOE_OK) return bad;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n = T * k, nbits = expert_bits(e_count);
  const int chunk = perm_chunk_pairs(n, e_count), nb = (n + chunk - 1) / chunk;
  int32_t* hist = static_cast<int32_t*>(ws);
  MOE_LAUNCH("permute_count", permute_count_kernel, dim3(nb), dim3(PERM_THREADS), 0, s, topk_idx, n, e_begin, e_count,
             nbits, chunk, hist);
  MOE_LAUNCH("permute_place", permute_place_kernel, dim3(nb), dim3(PERM_THREADS), 0, s, topk_idx, n, k, e_begin,
             e_count, nbits, chunk, static_cast<const int32_t*>(hist), expert_offsets, row_token, slot_row, topk_w,
             row_weight);
  if (xp) launch_rows(x, slot_row, T, d, k, xp, s);
  return moe_check_launch();
}
}  // namespace

// Stages 1-3 (and the Stage-4 gather if xp is given) in one call: the routing kernel counts its own
// winners per chunk of tokens, so the pairs are read back once (by the placing kernel) instead of twice.
extern "C" int moe_route_permute(const float* logits, const moe_bf16* x, int T, int d, int E_total, int k,
                                 int renormalize, int e_begin, int e_count, int32_t* topk_idx, float* topk_w,
                                 int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row, float* row_weight,
                                 moe_bf16* xp, void* ws, size_t ws_bytes, void* stream) {
  if (!logits || !topk_w || !moe_aligned16(logits) || !moe_aligned16(topk_w)) return MOE_ERR_INVALID;
  if (row_weight && !moe_aligned16(row_weight)) return MOE_ERR_INVALID;
  const int bad = check_permute_args(x, topk_idx, T, d, E_total, k, e_begin, e_count, expert_offsets, row_token, slot_row,
                                     xp, ws, ws_bytes);
  if (bad != MOE_OK) return bad;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n = T * k, nbits = expert_bits(e_count);
  int32_t* hist = static_cast<int32_t*>(ws);
  int chunk = 0, nb = 0;
  if (!moe_launch_route_count(logits, T, E_total, k, renormalize != 0, e_begin, e_count, nbits, topk_idx, topk_w, hist,
                              ws_bytes / sizeof(int32_t), &chunk, &nb, s)) {
    const int r = moe_route(logits, T, E_total, k, renormalize, topk_idx, topk_w, stream);
    if (r != MOE_OK) return r;
    chunk = perm_chunk_pairs(n, e_count);
    nb = (n + chunk - 1) / chunk;
    MOE_LAUNCH("permute_count", permute_count_kernel, dim3(nb), dim3(PERM_THREADS), 0, s,
               static_cast<const int32_t*>(topk_idx), n, e_begin, e_count, nbits, chunk, hist);
  }
  MOE_LAUNCH("permute_place", permute_place_kernel, dim3(nb), dim3(PERM_THREADS), 0, s,
             static_cast<const int32_t*>(topk_idx), n, k, e_begin, e_count, nbits, chunk,
             static_cast<const int32_t*>(hist), expert_offsets, row_token, slot_row,
             static_cast<const float*>(topk_w), row_weight);
  if (xp) launch_rows(x, slot_row, T, d, k, xp, s);
  return moe_check_launch();
}

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
// moe_permute for callers that cannot provide a workspace: the [chunk][expert] count table
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
  // every table cell the placing kernel reads is written by the counting kernel of the same call first,
  // so nothing has to be cleared between calls
  return permute_impl(x, topk_idx, nullptr, T, d, E_total, k, e_begin, e_count, expert_offsets, row_token, slot_row,
                      nullptr, xp, ws, STATIC_WS_BYTES, stream);
}
