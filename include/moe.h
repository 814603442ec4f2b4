/*
 * libmoe -- C ABI of the MI355X (gfx950) mixture-of-experts hot path.
 *
 * One GPU's share of a dropless top-k routed SwiGLU MoE feed-forward layer, forward and
 * backward.  The paper names this path only in prose: tokens are routed to a sparse
 * subset of experts (Sec. 3.2.3), each expert is a SwiGLU block served by "MoE-specific
 * operations" (Sec. 3.2.5, Efficient Kernels), and the expert weights are three stacked
 * tensors gate_proj / up_proj / down_proj with the expert on dim 0 (App. B.6, the
 * expert-parallel plan listing).  The arithmetic below is the standard definition of
 * such a layer:
 *
 *     S(t)    = k experts with the largest logit z[t,:], ordered (logit desc, index asc)
 *     w[t,j]  = softmax(z[t,:])[e_j], divided by the sum over the k selected if renorm
 *     FFN_e x = W_down[e] ( silu(W_gate[e] x) * (W_up[e] x) ),  silu(g) = g / (1 + exp(-g))
 *     Y[t]    = sum_j w[t,j] FFN_{e_j}(X[t])
 *
 * Conventions shared by every entry point
 *   - Pointers are DEVICE pointers unless marked [host].  The caller owns all memory,
 *     including workspaces; the library allocates nothing, frees nothing and keeps no
 *     pointer after a call returns.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and return without synchronising.  No device-to-host copy happens inside.
 *   - Matrices are dense row-major with 16-byte aligned base addresses.
 *   - dtype selects the element type of activations and expert weights: MOE_F32 or
 *     MOE_BF16 (bf16 operands, fp32 accumulation, one rounding to bf16 on output).
 *     Router logits, combine weights and their gradients are always fp32; indices,
 *     counts, offsets and maps are int32.  P = T * k routed rows must fit in int32.
 *   - Weight layout: w_gate, w_up : [E, f, d];  w_down : [E, d, f]  (expert-major,
 *     out-features x in-features); gradients use the layout and dtype of their weight.
 *   - Every entry point validates its arguments on the host first; when it returns
 *     MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED or MOE_ERR_WORKSPACE nothing has been launched.
 *     MOE_ERR_HIP means a kernel launch itself was refused: the kernels of the call enqueued
 *     before it still run, none after it is launched, and the outputs are undefined.  An entry
 *     point clears the HIP runtime's last-error state of the calling thread when it starts to
 *     launch, so an error left behind by an unrelated earlier call is not reported here.
 *     moe_last_error() gives the reason.
 *   - Workspaces must be 16-byte aligned.
 *   - Limits: 1 <= k <= 64, k <= E <= 1024; d and f multiples of 8; sizes > 0 except
 *     that T (or P) may be 0, which is a no-op.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = 1, /* null / misaligned pointer, non-positive size, k > E            */
  MOE_ERR_UNSUPPORTED = 2, /* dtype or shape outside the limits listed above                 */
  MOE_ERR_WORKSPACE = 3,   /* workspace pointer null or smaller than *_workspace_bytes says  */
  MOE_ERR_HIP = 4          /* a launch failed; see moe_last_error()                          */
};

enum { MOE_F32 = 0, MOE_BF16 = 1 };

/* Library version, "major.minor.patch" ([host] static string). */
const char* moe_version(void);

/* Text of the last error on the calling thread ([host], owned by the library, valid until
 * the next failing call on this thread; empty string if none). */
const char* moe_last_error(void);

/* ---------------------------------------------------------------------------------------
 * Routing (Sec. 3.2.3: tokens are routed to their assigned experts).
 *
 * For each token t: the k experts with the largest logits[t,:] (ties to the lower expert
 * index; +0 and -0 compare equal; logits must be finite), in slot order (logit descending,
 * index ascending); combine weights = softmax over all E experts, renormalised over the k
 * selected when renorm != 0; counts[e] = number of (token, slot) pairs routed to e;
 * offsets = exclusive prefix sum of counts, offsets[E] = T*k.
 *
 *   logits   [T,E] f32 in     topk_idx [T,k] i32 out    topk_w  [T,k] f32 out
 *   counts   [E]   i32 out    offsets  [E+1] i32 out
 *   ws / ws_bytes: scratch of at least moe_route_topk_workspace_bytes(T,E,k) bytes.
 */
size_t moe_route_topk_workspace_bytes(int T, int E, int k);
int32_t moe_route_topk(const float* logits, int T, int E, int k, int renorm,
                       int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * Expert forward with 8-bit operands (a widening beyond the paper, which says "mixed precision" and no more: App. A,
 * Table 4 caption).  Format: OCP MXFP8 -- elements in OFP8 E4M3 (bias 7, largest magnitude 448, no infinities),
 * one E8M0 scale 2^(s-127) per 32 consecutive elements of the REDUCTION dimension; an entry is scale * element.
 *
 * moe_mx8_quantise: src [rows, K] bf16 (device, row-major, contiguous) -> codes [rows, K] uint8 and scales, both device.
 *   Per block: s = max(biased float32 exponent of max|v| - 8, 0) (= floor(log2 max|v|) - 8 + 127 clamped at 0; an
 *   all-zero block gets 0), element = v / 2^(s-127) rounded to nearest even in E4M3 and saturated at +-448.  The
 *   arithmetic is exact up to that one rounding.  Scales are packed four to a 32-bit word, laid out
 *   [K/128][rows]: byte j (little endian) of word (g, row) belongs to elements 128 g + 32 j .. + 31 of the row.
 *   K must be a multiple of 128.  NaN and infinite inputs are not supported (result unspecified, no fault).
 *
 * moe_grouped_gemm_swiglu_fwd_mx8 (SwiGLU expert of Sec. 3.2.5 on the stacked weights of App. B.6):
 *   G = x Wg[e]^T, U = x Wu[e]^T with fp32 accumulation of the exact products of the scaled elements;
 *   act = silu(G) * U in fp32, quantised along f as above straight from fp32 (never rounded to bf16);
 *   yp = act Wd[e]^T, fp32 accumulation, rounded to bf16 once.
 *   xq, xs: codes [T, d] and scales [d/128][T] of the layer input, read by token through pair_of_row [P]
 *     (P = T * k; row r is token pair_of_row[r] / k), or -- pair_of_row NULL -- codes [P, d], scales [d/128][P]
 *     in expert order (T = P, k = 1).
 *   wgq, wuq [E, f, d] codes with wgs, wus [d/128][E*f] scales; wdq [E, d, f] codes with wds [f/128][E*d] scales
 *     (each weight quantised as one matrix of E*f, resp. E*d, rows).
 *   offsets [E+1] as for moe_grouped_gemm_swiglu_fwd.
 *   actq [P, f] codes out, acts [f/128][P] scales out (input format of the second product), yp [P, d] bf16 out.
 *   d and f must be multiples of 128; T * d < 2^32 when rows are read by token.  ws, ws_bytes: device workspace of
 *   at least moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(P, d, f, E).
 * Errors as everywhere: INVALID_ARG / UNSUPPORTED / WORKSPACE mean nothing was launched.
 *
 * moe_grouped_gemm_down_mx8: the second product alone, yp = act Wd[e]^T, on activation codes and scales the caller
 *   supplies (actq [P, f] and acts [f/128][P] in, read only); everything else as above, same workspace size.
 */
int32_t moe_mx8_quantise(const void* src, int64_t rows, int K, void* codes, void* scales, void* stream);
int32_t moe_grouped_gemm_down_mx8(const void* actq, const void* acts, const void* wdq, const void* wds, int P, int d,
                                  int f, int E, const int32_t* offsets, void* yp, void* ws, size_t ws_bytes,
                                  void* stream);
size_t moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(int P, int d, int f, int E);
int32_t moe_grouped_gemm_swiglu_fwd_mx8(const void* xq, const void* xs, int T, int k, const int32_t* pair_of_row,
                                        const void* wgq, const void* wgs, const void* wuq, const void* wus,
                                        const void* wdq, const void* wds, int P, int d, int f, int E,
                                        const int32_t* offsets, void* actq, void* acts, void* yp, void* ws,
                                        size_t ws_bytes, void* stream);

/* moe_route_topk for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without ws), same
 * kernels, same results bit for bit.  The per-workgroup histogram rows live in a static device array
 * inside the library instead: moe_route_topk_noalloc_max_bytes() bytes (2 MiB) held by every GPU the
 * library runs on until the process ends.  A shape whose moe_route_topk_workspace_bytes(T,E,k) exceeds
 * that maximum is rejected with MOE_ERR_UNSUPPORTED and nothing is launched.  The call allocates and
 * frees nothing (the first call on a device only looks up the array's address).  All calls on one GPU
 * share the array: calls that may overlap on that GPU (different streams) race and must be ordered by
 * the caller; calls on the same stream are ordered by the stream.
 */
size_t moe_route_topk_noalloc_max_bytes(void);
int32_t moe_route_topk_noalloc(const float* logits, int T, int E, int k, int renorm,
                               int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets,
                               void* stream);

/* Counts and offsets of an assignment that is already known (rows that an expert-parallel
 * dispatch has delivered to this GPU, Sec. 3.2.3: one local expert id per row, k = 1):
 * counts[e] = #{p : topk_idx[p] == e}, offsets = exclusive prefix sum, offsets[E] = n_pairs.
 *   topk_idx [n_pairs] i32 in (values in [0,E)); counts [E], offsets [E+1] i32 out;
 *   ws of at least moe_expert_offsets_workspace_bytes(n_pairs, E) bytes.
 */
size_t moe_expert_offsets_workspace_bytes(int n_pairs, int E);
int32_t moe_expert_offsets(const int32_t* topk_idx, int n_pairs, int E, int32_t* counts,
                           int32_t* offsets, void* ws, size_t ws_bytes, void* stream);

/* Backward of the combine weights with respect to the logits, selection held fixed.
 *   renorm != 0:  dlogits[t,e_j] = w_j (dw_j - sum_m w_m dw_m), 0 for unselected experts
 *   renorm == 0:  dlogits[t,e]   = p_e (1[e in S] dw_e - sum_{m in S} p_m dw_m), p = softmax(logits)
 *   dw, topk_w [T,k] f32 in; topk_idx [T,k] i32 in; logits [T,E] f32 in (read only when
 *   renorm == 0, may be NULL otherwise); dlogits [T,E] f32 out, every element written.
 */
int32_t moe_route_topk_bwd(const float* dw, const float* topk_w, const int32_t* topk_idx,
                           const float* logits, int T, int E, int k, int renorm,
                           float* dlogits, void* stream);

/* ---------------------------------------------------------------------------------------
 * Permutation into expert-contiguous rows (the local half of the token dispatch of
 * Sec. 3.2.3).  Stable counting sort of the P = T*k pairs p = t*k+j by expert:
 *   row_of_pair[p] = offsets[e_p] + #{p' < p : e_p' = e_p},  pair_of_row = its inverse,
 *   xp[row_of_pair[t*k+j], :] = x[t, :]   (bit copy).
 *   x [T,d] in; topk_idx [T,k] in; offsets [E+1] in (as written by moe_route_topk, or the
 *   exclusive scan of the bincount of topk_idx for pre-routed rows with k = 1);
 *   xp [P,d] out; row_of_pair, pair_of_row [P] i32 out.
 * x and xp may both be NULL: only the two maps are written (for the *_gather calls below, which
 * read x by token and need no xp).
 */
size_t moe_permute_workspace_bytes(int T, int E, int k);
int32_t moe_permute(const void* x, int dtype, int T, int d, int E, int k,
                    const int32_t* topk_idx, const int32_t* offsets,
                    void* xp, int32_t* row_of_pair, int32_t* pair_of_row,
                    void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Grouped SwiGLU expert FFN (Sec. 3.2.5 SwiGLU; App. B.6 stacked expert weights).
 * For each expert e and its rows r in [offsets[e], offsets[e+1]):
 *   G = xp W_gate[e]^T,  U = xp W_up[e]^T,  act = silu(G) * U,  yp = act W_down[e]^T.
 *   xp [P,d] in; offsets [E+1] in (offsets[E] == P); act [P,f] out; yp [P,d] out;
 *   g_save, u_save [P,f] out, or both NULL when the caller will let the backward recompute.
 */
size_t moe_grouped_gemm_swiglu_fwd_workspace_bytes(int dtype, int P, int d, int f, int E);
int32_t moe_grouped_gemm_swiglu_fwd(const void* xp, const void* w_gate, const void* w_up,
                                    const void* w_down, int dtype, int P, int d, int f, int E,
                                    const int32_t* offsets, void* g_save, void* u_save,
                                    void* act, void* yp, void* ws, size_t ws_bytes, void* stream);

/* Backward of the grouped FFN.  Per expert:
 *   dA = dyp W_down[e];  dW_down[e] = dyp^T act;  dG = dA * U * silu'(G);  dU = dA * silu(G);
 *   dW_gate[e] = dG^T xp;  dW_up[e] = dU^T xp;  dxp = dG W_gate[e] + dU W_up[e].
 * All three weight gradients are overwritten (not accumulated); experts without rows get
 * zeros.  g_save / u_save may both be NULL: G and U are then recomputed from xp (act is
 * still required).  `have_saved` in the workspace query says which variant will be called.
 * The backward workspace holds [dG | dU] (2 P f elements), the recomputed G and U when nothing was
 * saved, the device-built schedules, and room for fp32 partial weight-gradient tiles of experts
 * whose rows are cut into several reduction chunks under skewed routing: at most 2 ceil(P / C)
 * slots of 2 f d floats with C = max(2048, ceil(P / 32) rounded up to 256) rows (64 slots at most;
 * with balanced routing none is touched).
 */
size_t moe_grouped_gemm_swiglu_bwd_workspace_bytes(int dtype, int P, int d, int f, int E, int have_saved);
int32_t moe_grouped_gemm_swiglu_bwd(const void* dyp, const void* xp, const void* g_save,
                                    const void* u_save, const void* act, const void* w_gate,
                                    const void* w_up, const void* w_down, int dtype, int P, int d,
                                    int f, int E, const int32_t* offsets, void* dxp, void* dw_gate,
                                    void* dw_up, void* dw_down, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * The same grouped FFN with the dispatch folded into the products (Sec. 3.2.3 dispatch, Sec. 3.2.5
 * fused kernels): the rows of an expert are read from the token-major matrices while the tiles are
 * loaded, so neither xp nor the expert-ordered output gradient dyp is ever written.  P == T*k;
 * row r stands for pair pair_of_row[r], i.e. token pair_of_row[r] / k with weight topk_w[pair_of_row[r]].
 * T * d * element size must stay below 4 GiB.
 *
 * Forward: exactly moe_grouped_gemm_swiglu_fwd applied to xp[r] = x[pair_of_row[r] / k].
 *   x [T,d] in; pair_of_row [P] in (from moe_permute); the rest as in moe_grouped_gemm_swiglu_fwd.
 *   topk_w [T,k] f32 in, or NULL.  Given, the combine weight is applied here instead of in the combine:
 *   act[r] = topk_w[pair] * silu(G) * U (scaled in fp32, rounded once) and yp[r] = act[r] W_down[e]^T
 *   = topk_w[pair] * FFN(x[token]), so that Y is moe_unpermute_combine_fwd of yp with NULL weights and the
 *   backward finds its operand topk_w * act already written (act_w below).  g_save, u_save stay unscaled.
 *
 * Backward: exactly moe_unpermute_combine_bwd followed by moe_grouped_gemm_swiglu_bwd, i.e. with
 * dyp[r] = topk_w[pair] * dy[token] never stored:
 *   dA = topk_w[pair] * (dy[token] W_down[e]);   dW_down[e] = dy[token]^T (topk_w[pair] * act);
 *   dtopk_w[pair] = <dy[token] W_down[e], act[r]>  ( = <dy[token], yp[r]> );
 *   dG, dU, dW_gate, dW_up, dxp as in moe_grouped_gemm_swiglu_bwd with xp[r] = x[token].
 *   dy, x [T,d] in; topk_w [T,k] f32 in; g_save, u_save [P,f] in, or both NULL (recomputed from x);
 *   act_w [P,f] in, or NULL: topk_w[pair] * act as the forward with topk_w wrote it into `act`; NULL: it is
 *   formed here and staged in the workspace (one more [P,f] store);
 *   dxp [P,d] out (moe_unpermute_combine_fwd with NULL weights turns it into dx); dw_* out;
 *   dtopk_w [T,k] f32 out (input of moe_route_topk_bwd).  act and yp are not needed.
 * For bf16, act is recomputed from the rounded G and U in fp32, and topk_w * act is rounded once.
 */
size_t moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes(int dtype, int P, int d, int f, int E);
int32_t moe_grouped_gemm_swiglu_fwd_gather(const void* x, int T, int k, const int32_t* pair_of_row,
                                           const float* topk_w,
                                           const void* w_gate, const void* w_up, const void* w_down,
                                           int dtype, int P, int d, int f, int E, const int32_t* offsets,
                                           void* g_save, void* u_save, void* act, void* yp,
                                           void* ws, size_t ws_bytes, void* stream);
size_t moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes(int dtype, int P, int d, int f, int E, int have_saved);
int32_t moe_grouped_gemm_swiglu_bwd_gather(const void* dy, const void* x, int T, int k, const float* topk_w,
                                           const int32_t* pair_of_row, const void* g_save,
                                           const void* u_save, const void* act_w, const void* w_gate, const void* w_up,
                                           const void* w_down, int dtype, int P, int d, int f, int E,
                                           const int32_t* offsets, void* dxp, void* dw_gate, void* dw_up,
                                           void* dw_down, float* dtopk_w, void* ws, size_t ws_bytes,
                                           void* stream);

/* ---------------------------------------------------------------------------------------
 * Weighted un-permute / combine (the return half of the dispatch of Sec. 3.2.3).
 *   y[t,:] = sum_{j<k} topk_w[t,j] * yp[row_of_pair[t*k+j], :]   (fp32 sum, j ascending)
 * topk_w == NULL means all weights 1: that is the backward of moe_permute
 * (dx[t] = sum_j dxp[row_of_pair[t*k+j]]).
 */
int32_t moe_unpermute_combine_fwd(const void* yp, int dtype, int T, int d, int k,
                                  const float* topk_w, const int32_t* row_of_pair,
                                  void* y, void* stream);

/* Backward of the combine:
 *   dyp[row_of_pair[t*k+j], :] = topk_w[t,j] * dy[t,:];   dw[t,j] = <dy[t,:], yp[row,:]>.
 *   dy [T,d], yp [P,d] in; dyp [P,d] out; dw [T,k] f32 out.
 */
int32_t moe_unpermute_combine_bwd(const void* dy, const void* yp, int dtype, int T, int d, int k,
                                  const float* topk_w, const int32_t* row_of_pair,
                                  void* dyp, float* dw, void* stream);

/* ---------------------------------------------------------------------------------------
 * Router linear: the bias-free gate that turns hidden states into the logits moe_route_topk
 * consumes, and its backward, so that the library covers the block from hidden states in
 * to hidden-state gradient out (Sec. 3.2.3 speaks of routing only; a linear gate is the reading).
 *   w_router [E, d] (row e = gate vector of expert e; same element type as x), device.
 *   logits[t, e] = <x[t, :], w_router[e, :]>, fp32 accumulation, fp32 output [T, E].
 * Backward for an upstream dlogits [T, E] f32 (e.g. from moe_route_topk_bwd):
 *   dw_router[e, :] = sum_t dlogits[t, e] x[t, :]           [E, d], element type of x, overwritten
 *   dx[t, :] (+)= sum_e dlogits[t, e] w_router[e, :]        [T, d]; accumulate != 0 adds to what
 *                                                           dx holds (the expert-path gradient)
 * For bf16 the logit gradient is rounded to bf16 once before the two products.
 * Limits: d, E > 0, E <= 1024; bf16 needs d and E multiples of 8 (MOE_ERR_UNSUPPORTED otherwise).
 * T == 0: nothing is read; dw_router is written as zeros.  Workspaces as for the other calls.
 */
size_t moe_router_logits_workspace_bytes(int dtype, int T, int d, int E);
int32_t moe_router_logits(const void* x, const void* w_router, int dtype, int T, int d, int E,
                          float* logits, void* ws, size_t ws_bytes, void* stream);
size_t moe_router_bwd_workspace_bytes(int dtype, int T, int d, int E);
int32_t moe_router_bwd(const float* dlogits, const void* x, const void* w_router, int dtype,
                       int T, int d, int E, int accumulate, void* dx, void* dw_router,
                       void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Launch hook for measurement and tracing harnesses (not part of the layer's arithmetic; the
 * hot path of Sec. 3.2.3 / 3.2.5 is what it observes).  When a hook is installed the library calls
 *     hook(name, 0, stream, user)   just before it enqueues kernel `name` on `stream`,
 *     hook(name, 1, stream, user)   just after,
 *     hook(name, 2, stream, user)   when entry point `name` ("moe_permute", ...) is about to enqueue
 *                                   its first kernel, and
 *     hook(name, 3, stream, user)   after it has enqueued its last,
 * on the calling thread of the entry point, so a harness can record its own events on that
 * stream around each kernel and around each entry point.  name is a [host] static string
 * ("ffn_gate_up", "combine_fwd", ...); stream is the hipStream_t the entry point was given.  The library itself creates no
 * events, allocates nothing and copies nothing for this.  hook == NULL removes the hook.
 * The hook must not call back into the library.  Installing or removing it while another
 * thread is inside an entry point is safe; that call may or may not see the new hook.
 */
typedef void (*moe_launch_hook_t)(const char* name, int phase, void* stream, void* user);
int32_t moe_set_launch_hook(moe_launch_hook_t hook, void* user);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
