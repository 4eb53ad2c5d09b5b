/*
 * moe.h -- C ABI of the MI355X (gfx950) MoE expert layer: one GPU's share of a Mixture-of-Experts layer,
 * forward and backward.
 *
 * The layer is the top-k gated set of expert FFNs of Section II-A, with the symbols of the paper's notation table (Section III-A: d = d_model,
 * E routed experts, E_s shared always-active experts, top-k routing, n_mat = 3 SwiGLU matrices, expert FFN
 * dimension d_ffn) and the weight shapes of its memory model (Section III-A: W_up, W_gate in R^{d x d_ffn},
 * W_down in R^{d_ffn x d}).  The flow is the per-layer flow of Section IV with the two all-to-alls removed
 * (one GPU, every expert local):  routing -> local pack -> expert -> local unpack + weighted combine.
 *
 * Derived sizes used below:  E' = E + E_shared expert ids,  K' = k + E_shared slots per token,
 * N = T * K' rows after the permutation, slot id s = t*K' + j.
 *
 * Conventions for every compute entry point
 *   - Every pointer except `const moe_shape*` is a DEVICE pointer owned by the caller.  bf16 tensors travel as
 *     uint16_t bit patterns.  All tensors are dense, row-major, and 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue work on it:
 *     they never allocate, free, or synchronise the host.  Scratch comes from the caller's workspace `ws`
 *     (at least moe_workspace_bytes(shape) bytes, 256-byte aligned); calls that share a workspace must be
 *     ordered on one stream.
 *   - Return value: a moe_status.  Argument checks (NULL pointers, shape limits, alignment, workspace size)
 *     run on the host before anything is launched; on any error nothing is enqueued and no output is touched.
 *   - Outputs are fully overwritten, except the weight gradients when `accumulate` is 1.
 *
 * Shape limits:  1 <= k <= E <= 1024,  E' <= 1024,  T >= 0 (T = 0 is a no-op returning MOE_OK),
 * T*K' < 2^31,  d_model and d_ffn positive multiples of 64 and at most 2^22 (the kernels address a tile's rows
 * with 32-bit byte offsets: 256 rows of a 2^22-element bf16 row pitch still fit).
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Problem statement of one layer (Section III-A notation).  renorm != 0: the k gate weights of a token are
 * divided by their sum. */
typedef struct {
  int32_t T;        /* tokens on this GPU (b*s of the paper, or incoming rows of an expert-parallel shard) */
  int32_t d_model;  /* d */
  int32_t d_ffn;    /* expert FFN intermediate dimension */
  int32_t E;        /* routed experts held by this GPU */
  int32_t k;        /* top-k */
  int32_t E_shared; /* shared (always-active) experts, ids E .. E+E_shared-1 */
  int32_t renorm;
} moe_shape;

typedef enum {
  MOE_OK = 0,
  MOE_ERR_NULL = -1,      /* a required pointer is NULL */
  MOE_ERR_SHAPE = -2,     /* shape outside the limits above */
  MOE_ERR_ALIGN = -3,     /* a pointer is not 16-byte aligned (workspace: 256) */
  MOE_ERR_WORKSPACE = -4, /* workspace smaller than moe_workspace_bytes() */
  MOE_ERR_RUNTIME = -5    /* a HIP launch failed; hipGetLastError() holds the cause */
} moe_status;

/* Host-only helpers. */
const char* moe_status_str(int status);
/* Bytes of scratch that any single call below may need for this shape (0 if the shape is invalid). */
size_t moe_workspace_bytes(const moe_shape* shape);
/* Library version, for the binding's sanity check. */
int moe_abi_version(void);

/* Per-launch timing for benchmarks (host side; off by default).  While enabled, every kernel the library
 * launches is bracketed by two HIP events recorded on the launch stream (this creates events, so it is not for
 * callers that must not allocate).  moe_profile_get synchronises on record i and returns the kernel's label
 * (a static string) and its elapsed milliseconds; moe_profile_reset drops all records.  Not thread-safe with
 * respect to concurrent compute calls on other threads beyond a mutex around the record list. */
int moe_profile_enable(int on);
int moe_profile_count(void);
int moe_profile_get(int i, const char** name, float* ms);
int moe_profile_reset(void);

/* Top-k softmax gating (Section II-A "learned gating function"; Section III-A symbols E, E_s, k).
 * Per token: p = softmax(logits[t, 0:E]) in fp32; the k largest LOGITS are selected (descending; equal
 * logits -> lower expert id first); topk_w[t,j] = p[idx], divided by the sum over the k selected when renorm.
 * Slots j = k..K'-1 are the shared experts: idx = E + (j-k), weight 1.
 *   logits     [T,E]  fp32  in
 *   topk_idx   [T,K'] int32 out
 *   topk_w     [T,K'] fp32  out
 *   probs_save [T,E]  fp32  out, may be NULL (needed by moe_route_topk_bwd when renorm == 0)
 * NaN logits give unspecified (but in-range) indices. */
int moe_route_topk(const moe_shape* shape, const float* logits, int32_t* topk_idx, float* topk_w,
                   float* probs_save, void* stream);

/* Derivative of the gate weights with respect to the logits (shared slots contribute nothing).
 * renorm: dlogits[t, idx_j] = w_j (dw_j - sum_i w_i dw_i), zero elsewhere.
 * else  : dlogits[t, m] = p_m ([m selected] dw_m - sum_j p_{idx_j} dw_j); probs_save must be non-NULL.
 *   dtopk_w [T,K'] fp32 in;  topk_idx, topk_w as produced by moe_route_topk;  dlogits [T,E] fp32 out. */
int moe_route_topk_bwd(const moe_shape* shape, const float* dtopk_w, const int32_t* topk_idx,
                       const float* topk_w, const float* probs_save, float* dlogits, void* stream);

/* The learned gating function's linear map (Section II-A): logits[t,e] = <x[t], w_router[e]>.  The paper does not
 * print the function; a bias-free linear map with one weight row per routed expert is the reading used here.
 * bf16 operands, fp32 accumulation, fp32 result.
 *   x [T,d] bf16 in;  w_router [E,d] bf16 in;  logits [T,E] fp32 out. */
int moe_router_fwd(const moe_shape* shape, const uint16_t* x, const uint16_t* w_router, float* logits,
                   void* ws, size_t ws_bytes, void* stream);

/* Derivative of moe_router_fwd:
 *   dx_router[t] = sum_e dlogits[t,e] w_router[e]     [T,d] bf16 out (one rounding)
 *   dw_router[e] = sum_t dlogits[t,e] x[t]            [E,d] fp32, overwritten (accumulate == 0) or added to
 * dlogits [T,E] fp32 in.  dlogits enters the matrix cores as a bf16 head plus a bf16 remainder (two products), i.e.
 * with 16 significand bits; the products accumulate in fp32.  dw_router is the sum, in a fixed order, of the partial
 * sums of up to 32 equal parts of the token range (deterministic). */
int moe_router_bwd(const moe_shape* shape, const uint16_t* x, const uint16_t* w_router, const float* dlogits,
                   uint16_t* dx_router, float* dw_router, int accumulate, void* ws, size_t ws_bytes, void* stream);

/* Local pack (the per-GPU half of the dispatch of Section III-B: b*s*k rows of d_model bf16 values grouped by
 * expert).  A stable counting sort of the slots by expert id:
 *   counts[e]      = number of slots routed to e                                   [E']   int32 out
 *   offsets        = exclusive prefix sum of counts, offsets[E'] = N               [E'+1] int32 out
 *   row_of_slot[s] = offsets[e] + #{s' < s : idx[s'] = e}  (e = idx[s])            [N]    int32 out
 *   slot_of_row    = inverse of row_of_slot                                        [N]    int32 out
 *   x_perm[r]      = x[slot_of_row[r] / K']  (bit copy)                            [N,d]  bf16  out
 * x [T,d] bf16 in; topk_idx [T,K'] int32 in, every id must lie in [0,E') (ids outside are a caller error;
 * they are clamped into range so that no access leaves the buffers, and the result is then unspecified).
 * The result is deterministic (no atomics decide an order).  x and x_perm may be NULL together to build the
 * maps only. */
int moe_permute(const moe_shape* shape, const uint16_t* x, const int32_t* topk_idx, uint16_t* x_perm,
                int32_t* counts, int32_t* offsets, int32_t* row_of_slot, int32_t* slot_of_row,
                void* ws, size_t ws_bytes, void* stream);

/* moe_permute for callers that cannot allocate device memory or bring a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without `ws`, same results bit for bit.  The
 * scratch (per-slot ranks, per-block histograms) is an 8 MiB array that lives in the library's device image on every
 * GPU for the life of the process, so the call allocates nothing.  Limits: T*K' <= 2^20 and
 * ceil(T*K'/1024) * E' <= 2^20, else MOE_ERR_WORKSPACE (nothing enqueued).  Every call on a GPU shares that GPU's
 * array: calls that may overlap on one GPU (different streams, different host threads) race and must be ordered
 * by the caller.  Nothing in the array has to survive between calls or start at zero. */
int moe_permute_noalloc(const moe_shape* shape, const uint16_t* x, const int32_t* topk_idx, uint16_t* x_perm,
                        int32_t* counts, int32_t* offsets, int32_t* row_of_slot, int32_t* slot_of_row, void* stream);

/* Derivative of the row copy: dx[t] = sum_j dx_perm[row_of_slot[t*K'+j]] (fp32 sum in slot order, one bf16
 * rounding).   dx_perm [N,d] bf16 in;  dx [T,d] bf16 out. */
int moe_permute_bwd(const moe_shape* shape, const uint16_t* dx_perm, const int32_t* row_of_slot,
                    uint16_t* dx, void* stream);

/* The same with one more addend per token (the router's term of dx when the layer is closed from x):
 * dx[t] = sum_j dx_perm[row_of_slot[t*K'+j]] + dx_addend[t], fp32 sum (slots in order, then the addend), one bf16
 * rounding.   dx_addend [T,d] bf16 in. */
int moe_permute_bwd_add(const moe_shape* shape, const uint16_t* dx_perm, const int32_t* row_of_slot,
                        const uint16_t* dx_addend, uint16_t* dx, void* stream);

/* Expert FFNs over the ragged per-expert row segments (Section III-A: three matrices per expert, SwiGLU;
 * per-expert token counts s_e).  For expert e over rows [offsets[e], offsets[e+1]):
 *   G = X W_gate[e],  U = X W_up[e],  H = silu(G) * U,  Y = H W_down[e],   silu(z) = z / (1 + exp(-z)).
 * bf16 operands, fp32 accumulation; G, U, H, Y are each rounded to bf16 once.
 *   x_perm [N,d] bf16 in;  offsets [E'+1] int32 in (device; never read by the host)
 *   w_gate, w_up [E',d,f] bf16 in;  w_down [E',f,d] bf16 in
 *   y_perm [N,d] bf16 out;  save_g, save_u [N,f] bf16 out (the activations backward needs; together with
 *   x_perm this is the 3*d_ffn + d_model values per row of the paper's activation-memory model).  save_g and
 *   save_u may be NULL together: G and U then live in the workspace only (checkpointed forward, to be followed by
 *   moe_grouped_ffn_bwd_recompute)
 * Experts with no rows cost nothing and touch nothing. */
int moe_grouped_ffn_fwd(const moe_shape* shape, const uint16_t* x_perm, const int32_t* offsets,
                        const uint16_t* w_gate, const uint16_t* w_up, const uint16_t* w_down,
                        uint16_t* y_perm, uint16_t* save_g, uint16_t* save_u,
                        void* ws, size_t ws_bytes, void* stream);

/* Backward of moe_grouped_ffn_fwd.  Per expert e over its rows:
 *   dH = dY W_down[e]^T;  dW_down[e] = H^T dY;  dG = dH * U * silu'(G);  dU = dH * silu(G);
 *   dW_gate[e] = X^T dG;  dW_up[e] = X^T dU;  dX = dG W_gate[e]^T + dU W_up[e]^T.
 *   dy_perm [N,d] bf16 in;  save_g, save_u as written by the forward call
 *   dx_perm [N,d] bf16 out
 *   dw_gate, dw_up [E',d,f] fp32, dw_down [E',f,d] fp32: overwritten when accumulate == 0 (experts without
 *   rows get zeros), added to when accumulate == 1 (experts without rows are left untouched). */
int moe_grouped_ffn_bwd(const moe_shape* shape, const uint16_t* dy_perm, const uint16_t* x_perm,
                        const int32_t* offsets, const uint16_t* w_gate, const uint16_t* w_up,
                        const uint16_t* w_down, const uint16_t* save_g, const uint16_t* save_u,
                        uint16_t* dx_perm, float* dw_gate, float* dw_up, float* dw_down, int accumulate,
                        void* ws, size_t ws_bytes, void* stream);

/* The same backward without saved activations (the selective activation checkpointing used for the full-model
 * training runs of Section VII-B; in the activation-memory model of Section III-A the layer's share then drops to
 * d_model values per row): G and U are recomputed from x_perm with the forward's own kernel (4*d*f extra FLOP per row, bit-identical
 * to what forward produced), then everything is as in moe_grouped_ffn_bwd. */
int moe_grouped_ffn_bwd_recompute(const moe_shape* shape, const uint16_t* dy_perm, const uint16_t* x_perm,
                                  const int32_t* offsets, const uint16_t* w_gate, const uint16_t* w_up,
                                  const uint16_t* w_down, uint16_t* dx_perm, float* dw_gate, float* dw_up,
                                  float* dw_down, int accumulate, void* ws, size_t ws_bytes, void* stream);

/* Local unpack + weighted combine (the per-GPU half of the combine of Section III-B):
 *   out[t] = sum_{j<K'} topk_w[t,j] * y_perm[row_of_slot[t*K'+j]]   (fp32 accumulate in slot order, one bf16
 *   rounding).   y_perm [N,d] bf16 in;  row_of_slot [N] int32 in;  topk_w [T,K'] fp32 in;  out [T,d] bf16. */
int moe_unpermute_combine(const moe_shape* shape, const uint16_t* y_perm, const int32_t* row_of_slot,
                          const float* topk_w, uint16_t* out, void* stream);

/* Derivative of the combine:
 *   dy_perm[row_of_slot[s]] = bf16( topk_w[s] * dout[t(s)] );   dtopk_w[t,j] = <dout[t], y_perm[row]> (fp32).
 *   dout [T,d] bf16 in;  dy_perm [N,d] bf16 out;  dtopk_w [T,K'] fp32 out. */
int moe_unpermute_combine_bwd(const moe_shape* shape, const uint16_t* dout, const uint16_t* y_perm,
                              const int32_t* row_of_slot, const float* topk_w, uint16_t* dy_perm,
                              float* dtopk_w, void* stream);

/* ---- The single-GPU steps of the hierarchical all-to-all (Section V, Algorithm 1).  One rank's send buffer S has
 * N = num_nodes * R rows (R ranks per node) of row_bytes bytes (a multiple of 16; any element type): row n*R + l goes
 * to local rank l of node n.  M = num_nodes - 1; "the i-th remote node" counts the nodes other than node_id in
 * increasing order.  All pointers are device pointers, 16-byte aligned; the exchanges between ranks are the caller's. */

/* Phase 2 pack: F2s[i*R + r] = S[n_i*R + r] for every remote node n_i.   S [N rows] in;  F2s [M*R rows] out. */
int moe_halo_pack_remote(const void* S, void* F2s, int num_nodes, int R, size_t row_bytes, int node_id, void* stream);

/* Phase 3 repack: the received [M, R, row] buffer becomes [R, M, row]: F3s[r*M + i] = F2r[i*R + r], so that row block
 * r holds everything the remote nodes sent for local rank r.   F2r [M*R rows] in;  F3s [R*M rows] out. */
int moe_halo_repack(const void* F2r, void* F3s, int M, int R, size_t row_bytes, void* stream);

/* Final placement: O[node_id*R + r] = P1[r] (phase 1 result) and O[n_i*R + p] = F3r[p*M + i] (phase 3 result).
 *   P1 [R rows] in;  F3r [R*M rows] in (may be NULL when num_nodes == 1);  O [N rows] out. */
int moe_halo_unpack(const void* P1, const void* F3r, void* O, int num_nodes, int R, size_t row_bytes, int node_id,
                    void* stream);

/* ---- Load balancing through expert migration (Section VI).  Host functions on host arrays; nothing here touches
 * the GPU.  A placement is `groups[n_groups][n_experts / n_groups]`: the expert ids hosted by each GPU of an
 * expert-parallel group, every expert exactly once (else MOE_ERR_SHAPE). */

/* Running per-expert token counts (the load history an external scheduler inspects between steps):
 * running[e] += counts[e], counts being a host copy of what moe_permute wrote. */
int moe_load_accumulate(int64_t* running, const int32_t* counts, int n_experts);

/* ratio = max_k s_k / mean_k s_k with s_k the summed load of group k (1 = balanced): the quantity an external
 * scheduler compares with its threshold before it asks for a rebalancing. */
int moe_load_imbalance(const int64_t* load, int n_experts, int n_groups, const int32_t* groups, double* ratio);

/* The swap rebalancer of Section VI, Algorithm 2.  Up to max_iters times (the paper uses 100): take the
 * group with the largest summed load and the one with the smallest (first one on ties); among all exchanges of one
 * expert of the former with one of the latter take the one that reduces the difference of the two sums the most
 * (first one on ties; it must reduce it), exchange the two experts in place, and stop when none does.
 *   load [n_experts] int64 in (>= 0);  groups in/out;  n_swaps out;  swaps [2*max_iters] int32 out, may be NULL:
 *   the pairs (expert that left the heavy group, expert that left the light group) in the order performed. */
int moe_rebalance_experts(const int64_t* load, int n_experts, int n_groups, int32_t* groups, int max_iters,
                          int32_t* n_swaps, int32_t* swaps);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
