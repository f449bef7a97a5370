/*
 * xmoe.h - C ABI of libxmoe: the single-GPU hot path of the padding-free MoE layer of X-MoE
 * (arXiv 2508.13337) as hand-written HIP kernels for gfx950 (MI355X).
 *
 * The entry points follow the functions of the paper's Listing 1 ("Padding-free MoE-layer"):
 *     gating()            -> xmoe_gate_logits + xmoe_route
 *     PFT_construction()  -> xmoe_build_eri            (dropless: B = T*k rows)
 *     dispatch()          -> xmoe_dispatch             (the gather kernel; the all-to-alls are identity on one GPU)
 *     mlp()               -> xmoe_expert_ffn_fwd       (the "sequential GeMM" as one ragged grouped GEMM)
 *     combine()           -> xmoe_combine              (the scatter kernel, as an atomics-free gather-reduce)
 * and their backward companions (the paper only says backward mirrors forward, Section 4.3).
 *
 * Conventions that hold for every call
 *   - Every pointer except `stream` is a DEVICE pointer owned by the caller; the library never allocates,
 *     frees or synchronises (the xmoe_prof_* read-outs below excepted).  All work is enqueued on the hipStream_t passed as `void* stream` (NULL = the
 *     null stream).  Sizes are host integers.  Matrices are row-major and dense.
 *   - `dt` is the storage type of activations and weights: XMOE_F32 (4 bytes) or XMOE_BF16 (2 bytes).
 *     All arithmetic accumulates in float32; results are rounded once (nearest-even) when stored as bf16.
 *     Logits, probabilities, combine weights and their gradients are always float32; indices are int32.
 *   - Notation: T tokens, d model width (paper: S, H), E experts, k experts per token, f expert FFN width
 *     (paper: H_FFN), B = T*k routed rows.
 *   - Scratch memory comes from a caller-provided workspace of at least xmoe_workspace_bytes(...) bytes,
 *     256-byte aligned.  Its contents are undefined after the call.
 *   - Return value: an xmoe_status.  Argument errors are detected on the host before anything is enqueued
 *     (XMOE_ERR_INVALID_ARG, XMOE_ERR_UNSUPPORTED, XMOE_ERR_WORKSPACE); a failed launch gives XMOE_ERR_HIP.
 *   - Inputs must be finite; behaviour on NaN/Inf logits is unspecified.  Index arrays handed to a call must
 *     be the ones an earlier call of this library produced for the same sizes (they are not re-validated on
 *     the device).
 *   - Process-wide state.  No call depends on an earlier call's arguments, and calls on different streams share no
 *     device memory beyond what the caller passes (xmoe_build_eri_static excepted, see there).  What the library does
 *     keep per process, all of it host-side and none of it synchronised (the first call on a device, xmoe_prof_* and
 *     any other call must not race with each other from different threads):
 *       - per device, set on the first expert-MLP call there: the compute-unit count (size of the persistent grids)
 *         and the raised dynamic-LDS limit of the matrix-core kernels;
 *       - the event profiler of xmoe_prof_* (off by default).  Only while it is enabled do the matrix-core kernels
 *         also write their clock samples into a device-global table, which launches on different streams then share;
 *       - one environment variable, read once: XMOE_BWD_MERGE = 0 runs the last three GEMMs of the expert MLP's
 *         backward (dXd and the two weight gradients) as three launches instead of one (for comparisons and
 *         per-kernel profiles; the results are the same bits).
 */
#ifndef XMOE_H
#define XMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XMOE_OK = 0,
    XMOE_ERR_INVALID_ARG = 1,   /* null required pointer, size out of range, k > E, T*k >= 2^31, ... */
    XMOE_ERR_UNSUPPORTED = 2,   /* unknown dtype, E beyond the routing kernels' limit */
    XMOE_ERR_WORKSPACE = 3,     /* workspace missing, misaligned or too small */
    XMOE_ERR_HIP = 4            /* the HIP runtime reported an error at launch */
} xmoe_status;

typedef enum { XMOE_F32 = 0, XMOE_BF16 = 1 } xmoe_dtype;

/* `op` of xmoe_workspace_bytes */
typedef enum {
    XMOE_WS_BUILD_ERI = 0,      /* rows = T           */
    XMOE_WS_FFN_FWD = 1,        /* rows = B (FFN rows) */
    XMOE_WS_FFN_BWD = 2,        /* rows = B            */
    XMOE_WS_GATE_BWD = 3,       /* rows = T            */
    XMOE_WS_BUILD_ERI_CAPPED = 4, /* rows = T          */
    XMOE_WS_MLP2_FWD = 5,       /* rows = B            */
    XMOE_WS_MLP2_BWD = 6,       /* rows = B            */
    XMOE_WS_RBD_STAGE0 = 7      /* rows = T            */
} xmoe_ws_op;

/* activation of the two-matrix expert (xmoe_expert_mlp2_fwd / _bwd) */
typedef enum {
    XMOE_ACT_IDENTITY = 0,      /* act(h) = h: Listing 1's mlp() exactly as printed */
    XMOE_ACT_GELU = 1,          /* act(h) = h * Phi(h), the exact (erf) form        */
    XMOE_ACT_SILU = 2           /* act(h) = h * sigmoid(h)                          */
} xmoe_act;

/* Largest expert count the routing / ERI kernels accept. */
#define XMOE_MAX_EXPERTS 512

/* Human-readable name of a status code (static storage). */
const char* xmoe_status_string(int status);

/* Library version string (static storage). */
const char* xmoe_version(void);

/* Bytes of workspace the given call needs.  Host-only, pure.  Returns 0 for an unknown op. */
size_t xmoe_workspace_bytes(int op, int rows, int d, int E, int k, int f, int dt);

/* ---------------------------------------------------------------------------------------------------------
 * Gating, part 1 (Listing 1 gating(): "FFN(tokens)"; Appendix B.3: [S,H] tokens projected to [S,E] logits).
 *   logits[t,e] = sum_i x[t,i] * w_router[i,e] (+ bias[e])
 * evaluated in float32 in a fixed order, so that the top-k decision is reproducible bit for bit:
 *   64 partial sums, partial l taking i = l, l+64, ... in ascending i with one fused multiply-add per term from
 *   +0.0f; the partials folded by halving (offsets 32,16,8,4,2,1: p[l] += p[l+off]); then + bias[e].
 * x [T,d] dt; w_router [d,E] dt; bias [E] float32 or NULL; logits [T,E] float32 (out).
 */
int xmoe_gate_logits(const void* x, const void* w_router, const float* bias, float* logits,
                     int T, int d, int E, int dt, void* stream);

/* Gating, part 2 (Listing 1 gating(): softmax over E, then top-k).
 *   p = softmax(logits[t,:]);  slot j of token t holds the expert with the j-th largest logit, the lower index
 *   winning ties;  topk_w[t,j] = p[t, topk_idx[t,j]]  (raw probabilities, not renormalised).
 * logits [T,E] float32; topk_idx [T,k] int32 (out); topk_w [T,k] float32 (out).  1 <= k <= E <= XMOE_MAX_EXPERTS.
 */
int xmoe_route(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w, void* stream);

/* PFT construction (Listing 1 PFT_construction(), step 1 and the histogram; Section 4.1.1 defines the
 * ERI-arrays).  Stable counting sort of the T*k flat entries n = t*k + j by expert id; row i of the PFT is the
 * i-th entry of that order.  Dropless (max_token_count >= T), so B = T*k.
 *   token_ids[i]        token of row i (n / k)                    [B] int32
 *   expert_ids[i]       expert of row i (non-decreasing)          [B] int32
 *   combine_weights[i]  topk_w of row i's entry                   [B] float32
 *   tokens_per_expert   segment lengths                           [E] int32
 *   expert_offsets      exclusive prefix sum of the above, [E+1]  (expert e owns rows [off[e], off[e+1]))
 *   row_of_slot[n]      row that flat entry n landed in (inverse permutation)  [T*k] int32
 * ws: XMOE_WS_BUILD_ERI bytes.
 */
int xmoe_build_eri(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                   int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                   int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot,
                   void* ws, size_t ws_bytes, void* stream);

/* xmoe_build_eri for callers that cannot allocate device memory or size a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results as xmoe_build_eri (bit for
 * bit); the chunk histograms that xmoe_build_eri keeps in the caller's workspace live in a static device array of
 * XMOE_STATIC_ERI_SCRATCH_BYTES that the library holds on every GPU it runs on until the process ends.  Sizes whose
 * histograms do not fit - ceil(T*k / 1024) * E * 4 bytes > XMOE_STATIC_ERI_SCRATCH_BYTES - are rejected with
 * XMOE_ERR_WORKSPACE before anything is enqueued.  The call allocates nothing and frees nothing (the array's device
 * address is looked up once per device, on the first call there).  All calls on one GPU share that GPU's array: two
 * calls that overlap in time on one GPU (different streams, different threads) race on it and give undefined results;
 * calls that follow each other on one stream, or are otherwise ordered, are fine - nothing in the array has to start
 * at zero, every entry is written before it is read.
 */
#define XMOE_STATIC_ERI_SCRATCH_BYTES (1 << 20)
int xmoe_build_eri_static(const int32_t* topk_idx, const float* topk_w, int T, int E, int k,
                          int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                          int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot, void* stream);

/* PFT construction with token dropping (Listing 1 PFT_construction(), step 2; Appendix B.2): as xmoe_build_eri,
 * but every expert keeps at most max_token_count of the rows routed to it - those with the largest combine
 * weights; among equal weights the lower flat entry n = t*k + j is kept first; retained rows keep the order they
 * have in the dropless table.  The decision compares the float32 bit patterns of topk_w; no arithmetic is involved.
 * The number of retained rows B_kept <= T*k exists on the device only:
 *   tokens_per_expert[e] = min(rows routed to e, max_token_count);  expert_offsets[E] = B_kept;
 *   rows [B_kept, T*k): token_ids = -1, expert_ids = E, combine_weights = 0;  row_of_slot[n] = -1 for a dropped entry.
 * The other entry points run unchanged on such a table with T*k as the row count: xmoe_dispatch skips rows whose
 * token id is -1, xmoe_combine / xmoe_dispatch_bwd skip entries whose row is -1, xmoe_combine_bwd writes dw = 0 for
 * them, and the expert MLP takes its rows from expert_offsets.  max_token_count >= T reproduces xmoe_build_eri.
 * ws: XMOE_WS_BUILD_ERI_CAPPED bytes.
 */
int xmoe_build_eri_capped(const int32_t* topk_idx, const float* topk_w, int T, int E, int k, int max_token_count,
                          int32_t* tokens_per_expert, int32_t* expert_offsets, int32_t* token_ids,
                          int32_t* expert_ids, float* combine_weights, int32_t* row_of_slot,
                          void* ws, size_t ws_bytes, void* stream);

/* Shared experts behind a PFT whose row count only the device knows.  Shared experts (every token, weight 1) run as
 * n_shared further experts of the expert-MLP calls, their segments directly behind the PFT's rows.  Without token
 * dropping those rows are constants the caller can write once (the PFT has T*k rows).  After xmoe_build_eri_capped the
 * PFT ends at expert_offsets[E] = B_kept, so this call continues the arrays on the device:
 *   expert_offsets[E+1+s] = B_kept + (s+1)*T            (expert_offsets must have room for E + 1 + n_shared entries)
 *   token_ids[B_kept + s*T + t] = t,  combine_weights[B_kept + s*T + t] = 1     (room for T*k + n_shared*T entries)
 * xmoe_combine / xmoe_dispatch_bwd then find the shared rows through shared_row0 = &expert_offsets[E].
 */
int xmoe_append_shared_segments(int32_t* expert_offsets, int32_t* token_ids, float* combine_weights, int T, int E,
                                int n_shared, void* stream);

/* Redundancy-Bypassing Dispatch, stage 0 (Section 4.2 "Pilot Selection and Instantiation"), the metadata part.
 * Experts live on nodes in contiguous blocks: node(e) = e / experts_per_node.  A group is the set of one token's
 * flat entries n = t*k + j whose experts share a destination node (all tokens of a PFT share the source).  The
 * group's pilot is the entry with the smallest (rand_key[n], n) - rand_key [T*k] uint32 carries the random draws
 * the section asks for, made by the caller; every other entry of the group is a local replica.  Both groups get
 * ERI-arrays of their own that keep the PFT's order (sorted by expert, ascending token inside an expert):
 *   pilot_token_ids, pilot_expert_ids [T*k]     first n_pilot entries valid, then token -1 / expert E
 *   pilot_tokens_per_expert [E], pilot_offsets [E+1]       (pilot_offsets[E] = n_pilot, on the device only)
 *   replica_token_ids, replica_expert_ids [T*k], replica_tokens_per_expert [E], replica_offsets [E+1]   likewise
 *   s1_mapping_indices [T*k]   for replica r: position of its pilot inside the pilot segment of the pilot's expert
 *                              (the section's relative index, valid before and after the uneven exchange)
 *   s1_mapping_experts [T*k]   for replica r: the pilot's expert (E behind the last replica)
 *   merge_src [T*k]            for PFT row i: its row in the concatenation [pilot buffer ; replica buffer]
 * Inputs: topk_idx [T,k]; token_ids, expert_ids [T*k], expert_offsets [E+1], row_of_slot [T*k] of the dropless PFT
 * (xmoe_build_eri).  The pilot token buffer itself is xmoe_dispatch(x, pilot_token_ids); the replicas are rebuilt at
 * the destination as xmoe_dispatch(pilot buffer, absolute index), and the experts' input order as
 * xmoe_dispatch([pilot buffer ; replica buffer], merge_src).  ws: XMOE_WS_RBD_STAGE0 bytes.
 */
int xmoe_rbd_stage0(const int32_t* topk_idx, const uint32_t* rand_key, const int32_t* token_ids,
                    const int32_t* expert_ids, const int32_t* expert_offsets, const int32_t* row_of_slot, int T, int E,
                    int k, int experts_per_node, int32_t* pilot_token_ids, int32_t* pilot_expert_ids,
                    int32_t* pilot_tokens_per_expert, int32_t* pilot_offsets, int32_t* replica_token_ids,
                    int32_t* replica_expert_ids, int32_t* replica_tokens_per_expert, int32_t* replica_offsets,
                    int32_t* s1_mapping_indices, int32_t* s1_mapping_experts, int32_t* merge_src, void* ws,
                    size_t ws_bytes, void* stream);

/* Section 4.2: the relative pilot indices are re-encoded to absolute rows after the exchange:
 *   absolute[r] = pilot_offsets_at_destination[s1_mapping_experts[r]] + s1_mapping_indices[r]   (-1 for a sentinel)
 * n entries; pilot_offsets_at_destination [E+1] (on one device: pilot_offsets itself). */
int xmoe_rbd_absolute_index(const int32_t* s1_mapping_indices, const int32_t* s1_mapping_experts,
                            const int32_t* pilot_offsets_at_destination, int n, int E, int32_t* absolute,
                            void* stream);

/* Dispatch (Section 4.1.2 / Appendix B.4 gather kernel): xd[i,:] = x[token_ids[i],:], a bit copy.
 * x [T,d] dt; token_ids [B] int32 with values in [0,T); xd [B,d] dt (out).
 */
int xmoe_dispatch(const void* x, const int32_t* token_ids, int T, int B, int d, int dt, void* xd, void* stream);

/* Expert MLP (Listing 1 mlp(); Appendix B.4 "Sequential GeMM"): for each expert e and its rows
 * r in [expert_offsets[e], expert_offsets[e+1]):
 *   G = Xd_e Wg_e,  U = Xd_e Wu_e,  A = silu(G) * U,  Y_e = A Wd_e          (SwiGLU, no biases)
 * xd [B,d]; wg, wu [E,d,f]; wd [E,f,d] ("in x out"); expert_offsets [E+1] int32 on the device with
 * offsets[0] = 0 and offsets[E] = B.  Outputs: y [B,d]; g_save, u_save [B,f] (kept for backward).
 * An expert with no rows reads no weights.
 * row_index: NULL, or the gather of dispatch fused into the operand load (Section 3.2 / Table 2 names the dispatched copy
 * as one of the two activation tensors worth removing): xd is then the token matrix x [T,d] itself, row_index [B]
 * int32 holds token ids (token_ids of the ERI-arrays), and row i of the expert input is x[row_index[i]]; no [B,d]
 * copy of the tokens exists.  Entries of rows outside every segment are never read.  Results are bit-identical to
 * the call on the dispatched copy.  The token matrix reached through row_index (and the one reached through
 * dy_row_index in the backward call) may span at most 64 GiB: the matrix-core kernels address a gathered row with a
 * 32-bit offset in units of 16 bytes.  The calls do not know T and cannot check this.
 * Shared experts are served by the same call as E_s further experts whose segments are all T tokens: expert_offsets
 * continues with B+T, B+2T, ..., the weights of the shared experts follow the routed ones, and the rows are x again
 * (row_index continues with 0..T-1 per shared expert; or xmoe_dispatch makes the copies).  (A single call on x
 * itself with E = 1 and offsets {0,T} works too.)
 * ws: XMOE_WS_FFN_FWD bytes.
 */
int xmoe_expert_ffn_fwd(const void* xd, const int32_t* row_index, const int32_t* expert_offsets, int B, int E,
                        int d, int f, const void* wg, const void* wu, const void* wd,
                        void* g_save, void* u_save, void* y, int dt,
                        void* ws, size_t ws_bytes, void* stream);

/* Backward of the expert MLP (derived; A is recomputed from the saved G and U):
 *   dA = dY Wd^T;  dWd_e = A_e^T dY_e;  dG = dA * U * silu'(G);  dU = dA * silu(G);
 *   dXd = dG Wg^T + dU Wu^T;  dWg_e = Xd_e^T dG_e;  dWu_e = Xd_e^T dU_e.
 * xd, row_index: as in the forward call.
 * dy_row_index: NULL (dy is [B,d]), or the backward of combine fused into the operand loads, the mirror image of
 * row_index: dy is then the gradient of the layer's output, dout [T,d], dy_row_index [B] int32 holds token ids and
 * dy_row_scale [B] float32 (NULL = all 1) the combine weight of each row (token_ids and combine_weights of the
 * ERI-arrays; for a shared expert's rows 0..T-1 and 1), and row i of dY is dy_row_scale[i] * dout[dy_row_index[i]]:
 * no [B,d] gradient of the expert outputs exists.  The scale is applied in float32 behind the matrix product
 * (dA = s * (dout Wd^T), dWd = (s * A)^T dout), so the product s * dout is not rounded to dt first; results agree
 * with the call on a materialised dY to rounding.  Entries of rows outside every segment are never read.
 * dy_row_scale_grad: NULL, or [B] float32 (out): the gradient of the loss with respect to every row's scale,
 *   dy_row_scale_grad[i] = <row i of dY before the scale, Y[i]>,  Y[i] = A[i] Wd_e the expert's output for that row,
 * taken as sum_n (dY_unscaled[i] Wd^T)[n] * A[i,n] from the product the dAct GEMM forms anyway and the recomputed A,
 * in a fixed summation order.  With dy_row_index / dy_row_scale = token_ids / combine_weights this is the gradient
 * of the combine weights, row by row (xmoe_combine_bwd_weights puts it into slot order): Y, the second activation
 * tensor that Section 3.2 / Table 2 counts as held for backward (A_combine), then need not be kept after the
 * forward combine.  Entries of rows outside every segment are not written.
 * Outputs: dxd [B,d]; dwg, dwu [E,d,f]; dwd [E,f,d] - overwritten, all zero for an expert with no rows.
 * ws: XMOE_WS_FFN_BWD bytes.
 */
int xmoe_expert_ffn_bwd(const void* xd, const int32_t* row_index, const void* g_save, const void* u_save,
                        const void* dy, const int32_t* dy_row_index, const float* dy_row_scale,
                        float* dy_row_scale_grad, const int32_t* expert_offsets, int B, int E, int d, int f,
                        const void* wg, const void* wu, const void* wd,
                        void* dxd, void* dwg, void* dwu, void* dwd, int dt,
                        void* ws, size_t ws_bytes, void* stream);

/* The paper's own expert (Listing 1 mlp(pft, w1, w2): two sequential GeMMs over the ragged segments; Table 1 counts
 * 2 h' h parameters per expert and Table 3's totals need exactly two matrices).  For each expert e and its rows:
 *   H = Xd_e W1_e  (the listing's inter_activ),   A = act(H),   Y_e = A W2_e          (no biases)
 * The listing prints no activation between the two GeMMs while Section 3.2 (Table 2) counts two intermediate activations
 * between the FFN sub-layers, so `act` (an xmoe_act) is a parameter.
 * xd, row_index, expert_offsets, B, E, d, f: as in xmoe_expert_ffn_fwd.  w1 [E,d,f]; w2 [E,f,d] ("in x out").
 * Outputs: y [B,d]; h_save [B,f] (kept for backward).  ws: XMOE_WS_MLP2_FWD bytes.
 */
int xmoe_expert_mlp2_fwd(const void* xd, const int32_t* row_index, const int32_t* expert_offsets, int B, int E,
                         int d, int f, const void* w1, const void* w2, int act, void* h_save, void* y, int dt,
                         void* ws, size_t ws_bytes, void* stream);

/* Backward of the two-matrix expert (derived; A is recomputed from the saved H):
 *   dA = dY W2^T;  dW2_e = A_e^T dY_e;  dH = dA * act'(H);  dXd = dH W1^T;  dW1_e = Xd_e^T dH_e.
 * dy_row_index, dy_row_scale, dy_row_scale_grad: as in xmoe_expert_ffn_bwd.
 * Outputs: dxd [B,d]; dw1 [E,d,f]; dw2 [E,f,d] - overwritten, all zero for an expert with no rows.
 * ws: XMOE_WS_MLP2_BWD bytes.
 */
int xmoe_expert_mlp2_bwd(const void* xd, const int32_t* row_index, const void* h_save, const void* dy,
                         const int32_t* dy_row_index, const float* dy_row_scale, float* dy_row_scale_grad,
                         const int32_t* expert_offsets, int B, int E, int d, int f, const void* w1, const void* w2,
                         int act, void* dxd, void* dw1, void* dw2, int dt, void* ws, size_t ws_bytes, void* stream);

/* Combine (Section 4.1.2 / Appendix B.4 scatter kernel, which must accumulate since k rows share a token),
 * written as a gather-reduce so that no atomics are needed and the sum order is fixed:
 *   out[t,:] = sum_{j<k} topk_w[t,j] * y[row_of_slot[t*k+j],:]
 *              + sum_{s<n_shared} shared_rows[s*T + t,:]   (+ addend[t,:])
 * accumulated in float32 in this order, rounded once.  topk_w == NULL means all weights are 1 (this is then the
 * backward of dispatch).  shared_rows [n_shared*T, d] dt or NULL with n_shared = 0: outputs of experts that every
 * token visits with weight 1 (shared experts run as extra experts whose segment is all T tokens).
 * shared_row0: NULL, or a device pointer to one int32: shared_rows is then the base of a larger row buffer and the
 * shared experts' rows start at its row *shared_row0 (the row count of a capacity-limited PFT exists on the device
 * only, see xmoe_append_shared_segments).  addend [T,d] dt or NULL.
 */
int xmoe_combine(const void* y, const int32_t* row_of_slot, const float* topk_w, const void* shared_rows,
                 int n_shared, const int32_t* shared_row0, const void* addend, int T, int k, int d, int dt, void* out,
                 void* stream);

/* Backward of combine:
 *   dy[row_of_slot[t*k+j],:] = topk_w[t,j] * dout[t,:];     dw[t,j] = <dout[t,:], y[row_of_slot[t*k+j],:]>
 * dout [T,d]; y [B,d]; dy [B,d] (out); dw [T,k] float32 (out).
 * dy == NULL: only dw is computed (topk_w may then be NULL too) - for callers that hand dout, token ids and combine
 * weights to the expert MLP's backward instead (its dy_row_index), so that dY is never written.
 */
int xmoe_combine_bwd(const void* dout, const void* y, const int32_t* row_of_slot, const float* topk_w,
                     int T, int k, int d, int dt, void* dy, float* dw, void* stream);

/* The gradient of the combine weights from per-row inner products: dw[t,j] = row_grad[row_of_slot[t*k+j]], and 0 for
 * a dropped entry (row -1).  row_grad [B] float32 holds <dout[token of row i], y[i]> for every PFT row i
 * (dy_row_scale_grad of the expert MLP's backward); dw [T,k] float32 (out).  Together with that output it replaces
 * xmoe_combine_bwd in a layer that keeps neither dY nor Y.
 */
int xmoe_combine_bwd_weights(const float* row_grad, const int32_t* row_of_slot, int T, int k, float* dw, void* stream);

/* Backward of dispatch: dx[t,:] = sum_j dxd[row_of_slot[t*k+j],:] + sum_s shared_rows[s*T + t,:] (+ addend).
 * Same kernel as xmoe_combine with unit weights. */
int xmoe_dispatch_bwd(const void* dxd, const int32_t* row_of_slot, const void* shared_rows, int n_shared,
                      const int32_t* shared_row0, const void* addend, int T, int k, int d, int dt, void* dx,
                      void* stream);

/* Backward of softmax + top-k with the indices held constant:
 *   dp[t,e] = dw[t,j] if e == topk_idx[t,j] else 0;   dlogits = p * (dp - sum_e p*dp),  p = softmax(logits).
 * dlogits [T,E] float32 (out).
 */
int xmoe_route_bwd(const float* logits, const int32_t* topk_idx, const float* dw, int T, int E, int k,
                   float* dlogits, void* stream);

/* Backward of the gate projection:  dw_router = x^T dlogits  [d,E] dt;  dx_gate = dlogits w_router^T  [T,d] dt.
 * ws: XMOE_WS_GATE_BWD bytes.
 */
int xmoe_gate_logits_bwd(const void* x, const void* w_router, const float* dlogits, int T, int d, int E, int dt,
                         void* dw_router, void* dx_gate, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------------------
 * Optional per-kernel timing with HIP events on the caller's stream (for benchmarks).  Off by default.
 * While enabled, every kernel launch of the library is bracketed by a pair of events.  Not thread-safe.
 */
void xmoe_prof_enable(int on);
void xmoe_prof_reset(void);                       /* drop all recorded samples */
int xmoe_prof_num_kernels(void);                  /* number of kernel ids */
const char* xmoe_prof_kernel_name(int kernel_id); /* name of the __global__ function behind a kernel id */
/* Waits for all recorded events, then returns launches and total milliseconds of one kernel id. */
int xmoe_prof_get(int kernel_id, int* launches, double* total_ms);
/* Shader clock (GHz) that the last launch of a matrix-core kernel of the expert MLP ran at, measured by the kernel
 * itself (shader-clock counter against the constant 100 MHz counter over the lifetime of its first workgroup).
 * Synchronises with the device.  0 for a kernel id that keeps no such record or has not run. */
int xmoe_prof_shader_clock(int kernel_id, double* ghz);
/* A plain copy kernel, dst[0..bytes) = src[0..bytes): exactly `bytes` read and `bytes` written, the yardstick
 * that hardware byte counters are scaled by.  Device pointers, 16-byte aligned; bytes a multiple of 16; the
 * ranges must not overlap. */
int xmoe_prof_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* XMOE_H */
