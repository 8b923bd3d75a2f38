/*
 * moe_hotpath.h - C ABI of the MI355X (gfx950) SparseMoE expert hot path.
 *
 * The calls follow the five stages of the paper's FastSparseMoE block
 * (Section 3.1, Algorithm 1) for ONE GPU holding the local experts
 * [e_begin, e_begin + e_count) of an E-expert layer (e_count == E when there is
 * no expert parallelism):
 *
 *   moe_route                 Stage 1   Softmax + TopK of the router logits
 *   moe_permute               Stages 2-3 and the gather that opens Stage 4
 *   moe_grouped_gemm_fwd      Stage 4   three grouped products around Silu(gate)*up
 *   moe_unpermute_combine     Stage 5   ExpertOutputReductionForward
 *   moe_unpermute_combine_bwd Stage 5   ExpertOutputReductionBackward
 *   moe_grouped_gemm_bwd      derivative of Stage 4 (dgrad + wgrad; left to autograd in the paper)
 *   moe_permute_bwd           derivative of the Stage-4 gather
 *
 * Fused variants of the same stages: moe_grouped_gemm_fwd_gather / _bwd_gather (the products read the routed
 * rows of x themselves, no permuted copy), and moe_permute_gate, moe_grouped_gemm_fwd_folded,
 * moe_unpermute_sum, moe_grouped_gemm_bwd_folded (gate weights folded into the expert MLP: Stage 5 becomes a
 * plain sum and needs no backward pass of its own).  Stage 1's Router layer and the derivatives of Stage 1:
 * moe_router_fwd, moe_route_bwd, moe_router_bwd.
 *
 * Conventions, valid for every function below
 * -------------------------------------------
 * - Every pointer except `stream` is a DEVICE pointer to memory the caller owns,
 *   16-byte aligned, dense and row-major.  The library allocates nothing, frees
 *   nothing and never synchronises: all work is enqueued on `stream`
 *   (a hipStream_t passed as void*; NULL is the default stream).  Results are
 *   ready when the stream reaches them.  The only state the library keeps between
 *   calls is, per device, what it has looked up or configured once there (number of
 *   compute units, the kernels' LDS limit) and the benchmark facility at the end
 *   of this file.
 * - Outputs are overwritten, never accumulated into (weight gradients of
 *   experts without rows are written as zeros).
 * - Group sizes stay on the device (`expert_offsets`); no call reads them back.
 *   R_cap is the row capacity of the grouped buffers (T*k is always enough);
 *   rows at or beyond expert_offsets[e_count] are neither read nor written.
 * - moe_bf16 is a raw bfloat16 bit pattern.  Products accumulate in fp32; bf16
 *   results are rounded to nearest-even once, from the fp32 value.
 * - Return value: MOE_OK, or a negative MOE_ERR_* code.  Argument checks run on
 *   the host before anything is enqueued; a failed call enqueues nothing.
 *   Not checked (preconditions): logits finite; topk_idx values in [0, E) and
 *   distinct within a token; expert_offsets non-decreasing, starting at 0 and
 *   ending at most at R_cap.
 * - Calls on different streams may overlap as long as their buffers (including
 *   workspaces) do not.
 */
#ifndef MOE_HOTPATH_H
#define MOE_HOTPATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t moe_bf16;

enum {
  MOE_OK = 0,
  MOE_ERR_INVALID = -1,   /* null/misaligned pointer, non-positive or unsupported size */
  MOE_ERR_WORKSPACE = -2, /* workspace smaller than the matching *_workspace_bytes() */
  MOE_ERR_LAUNCH = -3     /* the HIP runtime refused a launch (hipGetLastError) */
};

/* Size limits (checked; MOE_ERR_INVALID beyond them):
 *   1 <= k <= E <= 512, e_count <= 512, d % 8 == 0, f % 8 == 0 for the row
 *   movers; the grouped products additionally need d % 64 == 0 and f % 64 == 0. */
#define MOE_MAX_EXPERTS 512

/* Library identification string (static storage). */
const char* moe_version(void);

/* Workspace sizes in bytes (host computation only). */
size_t moe_permute_workspace_bytes(int T, int k, int e_count);
size_t moe_grouped_gemm_bwd_workspace_bytes(int R_cap, int f);
/* Upper bound that is enough for any call on a layer of this shape with R_cap <= T*k and at most E local
 * experts: the largest of moe_permute_workspace_bytes(T, k, E), moe_grouped_gemm_bwd_workspace_bytes(T*k, f),
 * moe_grouped_gemm_bwd_folded_workspace_bytes(T*k, f) and moe_router_bwd_workspace_bytes(T, d, E).
 * 0 for a non-positive size or when T*k does not fit an int. */
size_t moe_workspace_bytes(int T, int E, int k, int d, int f);

/*
 * Stage 1 (Algorithm 1: probs = Softmax(logits); weights, indices = TopK(probs)).
 *   logits   [T, E] fp32
 *   topk_idx [T, k] int32  slot i holds the expert with the i-th largest logit;
 *                          equal logits go to the lower expert id (-0.0 == +0.0)
 *   topk_w   [T, k] fp32   softmax probability of each chosen expert; divided by
 *                          the sum over the k chosen ones when renormalize != 0
 *                          (renormalize == 0 is Algorithm 1 as printed)
 */
int moe_route(const float* logits, int T, int E, int k, int renormalize,
              int32_t* topk_idx, float* topk_w, void* stream);

/*
 * Stages 2-3 (token counting, index generation) and mlp_in = input[input_indices].
 * The (token, slot) pairs whose expert is local are grouped by expert; inside an
 * expert they keep token order (a stable counting sort, done without atomics, so
 * the result is unique and reproducible).
 *   x              [T, d] bf16
 *   topk_idx       [T, k] int32, values in [0, E_total)
 *   expert_offsets [e_count+1] int32  out: exclusive prefix sum of the per-expert
 *                                     row counts (Algorithm 1: cum_token_counts)
 *   row_token      [T*k] int32        out: token of each grouped row (input_indices);
 *                                     entries at or beyond R are left untouched
 *   slot_row       [T, k] int32       out: grouped row of pair (t, i), -1 when its
 *                                     expert is not local (dense form of
 *                                     output_indices / selected_expert_indices)
 *   xp             [T*k, d] bf16      out: xp[r] = x[row_token[r]] for r < R.
 *                                     May be NULL: then only the index arrays are
 *                                     produced and x is not read (for the *_gather
 *                                     products below, which read x through row_token)
 *   ws             at least moe_permute_workspace_bytes(T, k, e_count)
 */
int moe_permute(const moe_bf16* x, const int32_t* topk_idx,
                int T, int d, int E_total, int k, int e_begin, int e_count,
                int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row,
                moe_bf16* xp, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_permute without a workspace argument, for callers that cannot allocate device memory at all
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the histogram
 * table lives in a device array inside the library image, moe_permute_static_ws_capacity() bytes
 * (1 MiB) on every GPU the library is used on, held until the process ends.  Arguments and results are
 * exactly those of moe_permute.  A shape whose table does not fit
 * (moe_permute_workspace_bytes(T, k, e_count) > capacity) is refused with MOE_ERR_WORKSPACE and nothing
 * is enqueued.  The call allocates nothing and frees nothing.  Its first call on a device looks the
 * array's address up (no allocation, but do it before a graph capture begins).  All calls on one GPU
 * share that GPU's array: two such calls that overlap in time on one GPU (different streams) race;
 * calls on one stream, or ordered by events, are fine.
 */
size_t moe_permute_static_ws_capacity(void);
int moe_permute_static_ws(const moe_bf16* x, const int32_t* topk_idx,
                          int T, int d, int E_total, int k, int e_begin, int e_count,
                          int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row,
                          moe_bf16* xp, void* stream);

/* dx[t] = sum over the local slots i of token t of dxp[slot_row[t, i]] (fp32 sum
 * in slot order, rounded once); a token without local slot gets zeros.
 *   dxp [R_cap, d] bf16, slot_row [T, k] int32, dx [T, d] bf16 */
int moe_permute_bwd(const moe_bf16* dxp, const int32_t* slot_row, int T, int k, int d,
                    moe_bf16* dx, void* stream);

/*
 * Stage 4 (Algorithm 1: gate_out, up_out = Grouped_mm(mlp_in, gate/up_weight);
 * mul_out = Silu(gate_out) * up_out; mlp_out = Grouped_mm(mul_out, down_weight)).
 * For each local expert e with rows r in [expert_offsets[e], expert_offsets[e+1]):
 *   g[r] = xp[r] . Wg[e]^T,  u[r] = xp[r] . Wu[e]^T,  h[r] = silu(g[r]) * u[r],
 *   yp[r] = h[r] . Wd[e]^T.
 *   xp [R_cap, d]; Wg, Wu [E, f, d]; Wd [E, d, f]  (each expert's [out, in]
 *   weight, stacked over the E local experts); g, u, h [R_cap, f] are saved for
 *   the backward call; yp [R_cap, d].  All bf16; h is formed from the fp32
 *   accumulators, before g and u are rounded.
 */
int moe_grouped_gemm_fwd(const moe_bf16* xp, const int32_t* expert_offsets,
                         const moe_bf16* Wg, const moe_bf16* Wu, const moe_bf16* Wd,
                         int E, int R_cap, int d, int f,
                         moe_bf16* g, moe_bf16* u, moe_bf16* h, moe_bf16* yp, void* stream);

/*
 * Stage 4 with mlp_in = input[input_indices] folded into the first product: the
 * same results as moe_grouped_gemm_fwd on xp[r] = x[row_token[r]], but the gate/up
 * product loads the rows of x itself, so xp need not exist.
 *   x [T, d] bf16, T*d*2 bytes at most 4 GiB (row offsets are 32-bit);
 *   row_token [R_cap] int32 as written by moe_permute; everything else as above.
 */
int moe_grouped_gemm_fwd_gather(const moe_bf16* x, int T, const int32_t* row_token,
                                const int32_t* expert_offsets,
                                const moe_bf16* Wg, const moe_bf16* Wu, const moe_bf16* Wd,
                                int E, int R_cap, int d, int f,
                                moe_bf16* g, moe_bf16* u, moe_bf16* h, moe_bf16* yp, void* stream);

/*
 * Derivative of Stage 4.  With s = sigmoid(g):
 *   dh = dyp . Wd[e];  dg = dh * u * s * (1 + g * (1 - s));  du = dh * g * s;
 *   dxp = dg . Wg[e] + du . Wu[e];
 *   dWd[e] = dyp^T . h;  dWg[e] = dg^T . xp;  dWu[e] = du^T . xp   (zeros if e has no rows).
 *   dyp, xp, dxp [R_cap, d]; g, u, h [R_cap, f]; dWg, dWu [E, f, d]; dWd [E, d, f]; all bf16.
 *   ws at least moe_grouped_gemm_bwd_workspace_bytes(R_cap, f), 256-byte aligned.  On return it holds
 *   dg [R_cap, f] bf16 at ws and du [R_cap, f] bf16 at ws + (that size / 2) (rows below
 *   expert_offsets[E] written): a caller may read them, e.g. to check them.
 */
int moe_grouped_gemm_bwd(const moe_bf16* dyp, const moe_bf16* xp,
                         const moe_bf16* g, const moe_bf16* u, const moe_bf16* h,
                         const int32_t* expert_offsets,
                         const moe_bf16* Wg, const moe_bf16* Wu, const moe_bf16* Wd,
                         int E, int R_cap, int d, int f,
                         moe_bf16* dxp, moe_bf16* dWg, moe_bf16* dWu, moe_bf16* dWd,
                         void* ws, size_t ws_bytes, void* stream);

/* The same with xp[r] = x[row_token[r]] read through row_token by the two weight-gradient
 * products that need it (dWg, dWu); x, T, row_token as for moe_grouped_gemm_fwd_gather. */
int moe_grouped_gemm_bwd_gather(const moe_bf16* dyp, const moe_bf16* x, int T, const int32_t* row_token,
                                const moe_bf16* g, const moe_bf16* u, const moe_bf16* h,
                                const int32_t* expert_offsets,
                                const moe_bf16* Wg, const moe_bf16* Wu, const moe_bf16* Wd,
                                int E, int R_cap, int d, int f,
                                moe_bf16* dxp, moe_bf16* dWg, moe_bf16* dWu, moe_bf16* dWd,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * Stages 1-3 in one call (Algorithm 1: Softmax, TopK, token counting, index generation), and the Stage-4
 * gather if xp is given: the results of moe_route followed by moe_permute (or moe_permute_gate), bit for
 * bit, with one launch fewer: the routing kernel counts its own winners per local expert, so the pairs are
 * not read back to be counted.
 *   logits, topk_idx, topk_w, renormalize   as moe_route (both outputs are written in full)
 *   x, xp                                   as moe_permute; both may be NULL (index generation only)
 *   row_weight                              as moe_permute_gate, or NULL
 *   expert_offsets, row_token, slot_row, ws as moe_permute (a workspace beyond the minimum is put to use: the
 *                                           count table may then have more, shorter rows of tokens, which
 *                                           spares the routing kernel a second pass; the results do not change)
 */
int moe_route_permute(const float* logits, const moe_bf16* x, int T, int d, int E_total, int k, int renormalize,
                      int e_begin, int e_count, int32_t* topk_idx, float* topk_w,
                      int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row, float* row_weight,
                      moe_bf16* xp, void* ws, size_t ws_bytes, void* stream);

/*
 * The layer with the gate weights folded into the expert MLP (Stages 2-5 and their derivatives give the
 * same out, dx, dW and dgate; the gate-weighted sum of Stage 5 is linear, so the weight of a routed row
 * may multiply h instead of the expert's output).  Forward: moe_permute_gate, moe_grouped_gemm_fwd_folded,
 * moe_unpermute_sum.  Backward: moe_grouped_gemm_bwd_folded, moe_permute_bwd.  The backward then needs
 * neither yp nor the scaled output gradient dyp[r] = w_r dout[token_r]: no separate pass over [R, d] rows
 * computes dgate and dyp.
 *
 * moe_permute_gate: moe_permute without moving rows, plus the gate weight of every routed row:
 *   row_weight[slot_row[t, i]] = topk_w[t, i] for every local slot.  topk_w [T, k] fp32 (device),
 *   row_weight [R_cap] fp32 (device, written for rows below expert_offsets[e_count]); the rest as moe_permute.
 */
int moe_permute_gate(const int32_t* topk_idx, const float* topk_w, int T, int E_total, int k, int e_begin, int e_count,
                     int32_t* expert_offsets, int32_t* row_token, int32_t* slot_row, float* row_weight,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * moe_grouped_gemm_fwd_gather with hw = w_r * silu(g) * u in place of h (w_r = row_weight[r], applied to
 * the fp32 value before the one rounding to bf16) and therefore ypw = hw . Wd[e]^T = w_r * yp in place of yp.
 * g and u are as before.  row_weight [R_cap] fp32 (device); the rest as moe_grouped_gemm_fwd_gather.
 */
int moe_grouped_gemm_fwd_folded(const moe_bf16* x, int T, const int32_t* row_token, const float* row_weight,
                                const int32_t* expert_offsets,
                                const moe_bf16* Wg, const moe_bf16* Wu, const moe_bf16* Wd,
                                int E, int R_cap, int d, int f,
                                moe_bf16* g, moe_bf16* u, moe_bf16* hw, moe_bf16* ypw, void* stream);

/* out[t] = sum over local slots i, in slot order, of ypw[slot_row[t, i]] (fp32 sum, rounded once): Stage 5
 * for rows that already carry their gate weight.  Shapes as moe_unpermute_combine. */
int moe_unpermute_sum(const moe_bf16* ypw, const int32_t* slot_row, int T, int k, int d, moe_bf16* out, void* stream);

/*
 * Derivative of Stages 4 and 5 after moe_grouped_gemm_fwd_folded, from dout [T, d] itself.  With
 * t_r = row_token[r], w_r = row_weight[r], s = sigmoid(g):
 *   dh0 = dout[t_r] . Wd[e];  dgate[t, i] = sum_c dh0[r, c] * silu(g[r, c]) * u[r, c] for r = slot_row[t, i]
 *   (0 for a slot without local row; fp32: per 64-column strip in column order, strips added in order);
 *   dh = w_r * dh0;  dg, du, dxp, dWg, dWu as in moe_grouped_gemm_bwd (rows of x read through row_token);
 *   dWd[e] = dout[t_r]^T . hw   (rows of dout read through row_token).
 *   dout, x [T, d] bf16 (T*d*2 bytes at most 4 GiB); slot_row [T, k] int32; g, u, hw [R_cap, f] bf16;
 *   dgate [T, k] fp32; dxp [R_cap, d]; dWg, dWu [E, f, d]; dWd [E, d, f]; all device memory.
 *   ws at least moe_grouped_gemm_bwd_folded_workspace_bytes(R_cap, f): dg, du and the strips' partial sums.
 */
size_t moe_grouped_gemm_bwd_folded_workspace_bytes(int R_cap, int f);
int moe_grouped_gemm_bwd_folded(const moe_bf16* dout, const moe_bf16* x, int T, int k,
                                const int32_t* row_token, const float* row_weight, const int32_t* slot_row,
                                const moe_bf16* g, const moe_bf16* u, const moe_bf16* hw,
                                const int32_t* expert_offsets,
                                const moe_bf16* Wg, const moe_bf16* Wu, const moe_bf16* Wd,
                                int E, int R_cap, int d, int f,
                                moe_bf16* dxp, moe_bf16* dWg, moe_bf16* dWu, moe_bf16* dWd, float* dgate,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * Stage 5, ExpertOutputReductionForward:
 *   out[t] = sum over local slots i, in slot order, of topk_w[t, i] * yp[slot_row[t, i]]
 * (fp32 sum, rounded once); zeros for a token without local slot.
 *   yp [R_cap, d] bf16, slot_row [T, k] int32, topk_w [T, k] fp32, out [T, d] bf16
 */
int moe_unpermute_combine(const moe_bf16* yp, const int32_t* slot_row, const float* topk_w,
                          int T, int k, int d, moe_bf16* out, void* stream);

/*
 * Stage 5, ExpertOutputReductionBackward:
 *   dyp[slot_row[t, i]] = topk_w[t, i] * dout[t]
 *   dgate[t, i] = <yp[slot_row[t, i]], dout[t]>   (0 where slot_row[t, i] < 0)
 * dgate is the gradient with respect to the weights as used by the combine.
 *   dout [T, d] bf16, yp, dyp [R_cap, d] bf16, dgate [T, k] fp32
 */
int moe_unpermute_combine_bwd(const moe_bf16* dout, const moe_bf16* yp,
                              const int32_t* slot_row, const float* topk_w,
                              int T, int k, int d, moe_bf16* dyp, float* dgate, void* stream);

/*
 * The router itself and the derivative of Stage 1 (Algorithm 1: logits = Router(input), a Linear
 * layer; the paper leaves the backward pass to autograd).  These calls complete the layer as a
 * drop-in block: moe_router_fwd feeds moe_route, and dgate from moe_unpermute_combine_bwd goes
 * back through moe_route_bwd and moe_router_bwd.
 *
 * moe_router_fwd:  logits[t, e] = sum_j x[t, j] * Wr[e, j]   (no bias)
 *   x [T, d] bf16, Wr [E, d] fp32, logits [T, E] fp32 out.  d % 16 == 0, E <= MOE_MAX_EXPERTS.
 *   The products are formed exactly and summed in fp32 (the summation order differs from a host
 *   matrix product, so logits agree to fp32 rounding, not bit for bit).
 */
int moe_router_fwd(const moe_bf16* x, const float* Wr, int T, int d, int E, float* logits, void* stream);

/*
 * moe_route_bwd:  gradient with respect to the logits for given dgate[t, i] = dL/d topk_w[t, i],
 * the chosen experts held fixed.  With p = Softmax(logits), s_i = p[topk_idx[t, i]], S = sum_i s_i:
 *   renormalize != 0:  dL/ds_i = (dgate_i - sum_j dgate_j * s_j / S) / S ;  otherwise dL/ds_i = dgate_i
 *   dlogits[t, e] = p_e * (dL/dp_e - sum_i dL/ds_i * s_i),  dL/dp_e = dL/ds_i if e = topk_idx[t, i], else 0.
 *   logits [T, E] fp32, topk_idx [T, k] int32 (distinct per token), dgate [T, k] fp32,
 *   dlogits [T, E] fp32 out.
 */
int moe_route_bwd(const float* logits, const int32_t* topk_idx, const float* dgate, int T, int E, int k,
                  int renormalize, float* dlogits, void* stream);

/*
 * moe_router_bwd:  derivative of the Linear layer.
 *   dWr[e, j] = sum_t dlogits[t, e] * x[t, j]                  fp32 [E, d] out (overwritten)
 *   dx[t, j] += sum_e dlogits[t, e] * Wr[e, j]                 bf16 [T, d] IN-OUT: the router's share
 *     is ADDED to what dx holds (the expert path's gradient from moe_permute_bwd), in fp32, and the
 *     sum is rounded once.  This is the one argument of the library that is accumulated into.
 *   ws at least moe_router_bwd_workspace_bytes(T, d, E): partial sums of dWr over chunks of 256
 *   tokens, reduced in a fixed order (no atomics: results are reproducible).
 */
size_t moe_router_bwd_workspace_bytes(int T, int d, int E);
int moe_router_bwd(const moe_bf16* x, const float* Wr, const float* dlogits, int T, int d, int E,
                   moe_bf16* dx, float* dWr, void* ws, size_t ws_bytes, void* stream);

/*
 * Per-kernel timing for benchmarks (not part of the paper's method).  While
 * enabled, every kernel the library launches is bracketed by two HIP events
 * recorded on the launch stream.  moe_prof_read synchronises on the recorded
 * events and returns, for entry `index` (0 .. moe_prof_count()-1), the kernel's
 * name, its summed duration in milliseconds and its launch count.  These calls
 * create HIP events (host objects) and are not thread-safe; leave profiling off
 * in production.
 */
int moe_prof_enable(int on);        /* also clears what was recorded */
int moe_prof_count(void);
int moe_prof_read(int index, char* name, int name_cap, float* total_ms, int* launches);

/*
 * Matrix-pipe probe for benchmarks (not part of the paper's method): what rate of
 * v_mfma_f32_16x16x32_bf16 (the form the grouped products use) the chip sustains for given operand VALUES.  The clock
 * of the chip follows its power draw, which depends on how many operand bits
 * toggle, so the ceiling for real data lies below the published peak.
 *   a    [workgroups*512, 32] bf16, device: 4 activation fragments per lane
 *   b    [workgroups*512, 16] bf16, device: 2 weight fragments per lane
 *   sink [workgroups*512] f32, device, overwritten (keeps the loop alive)
 * Launches `workgroups` workgroups of 8 waves, each lane issuing 8*iters MFMAs on
 * its register-resident fragments with no memory traffic, waits for the kernel
 * (this call synchronises on its own events) and returns its duration in
 * milliseconds, its FLOP count and the core clock in GHz observed by wave 0.
 */
int moe_prof_mfma_ceiling(const moe_bf16* a, const moe_bf16* b, int workgroups, int iters, float* sink,
                          float* ms, double* flop, double* clock_ghz, void* stream);

/*
 * Memory probe for benchmarks (not part of the paper's method): a kernel that only reads.  `workgroups`
 * workgroups of 256 threads read the first bytes / 16384 whole 16 KB blocks of src (device, 16-byte aligned)
 * with 16-byte loads and write one word per thread to sink [workgroups * 256] (device).  Enqueued on
 * `stream` like any other call (timed through moe_prof_enable / moe_prof_read under the name
 * "stream_read"); the rate it reaches on buffers that no cache holds is what the row movers' rates
 * should be read against.
 */
int moe_prof_stream_read(const void* src, size_t bytes, uint32_t* sink, int workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HOTPATH_H */
