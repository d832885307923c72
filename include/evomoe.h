/*
 * evomoe.h -- C ABI of the MI355X (gfx950) DTS-Gate Mixture-of-Experts layer.
 *
 * The library implements the MoE layer of EvoMoE's gate-sparsify phase
 * (arXiv 2112.14397, Methods, Stage 2 and Algorithms 1-2):
 *
 *     g'(x_s) = softmax((x_s . W_g + b_g + zeta_s) / tau)          (Eq. gumbel_softmax)
 *     g(x_s)_i = g'(x_s)_i  if g'(x_s)_i > c  else 0               (Eq. adaptive_sparsity)
 *     y_s = sum_{i in Id_s} g(x_s)_i * e_i(x_s)                    (Eq. moe_weighted_sum_problem)
 *     e_i(x) = W2_i . act(W1_i . x + b1_i) + b2_i                  (Eq. ffn)
 *
 * forward and backward, on ONE GPU with all experts resident.
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Every tensor argument is a caller-owned DEVICE pointer (unless the
 *    parameter name ends in _host), row-major, densely packed, 16-byte
 *    aligned.  The library never frees or retains caller memory.
 *  - "elem" below means the layer's storage type shape->dtype (float or
 *    bfloat16).  Gate quantities (W_g, b_g, noise, g', weights, their
 *    gradients) and all biases / bias gradients are float32 regardless.
 *  - Symbols: T tokens, d model width (paper's D), E experts (paper's N),
 *    F expert hidden width, P = number of selected (token, expert) pairs,
 *    P_cap = capacity of every per-pair buffer (rows).  A "row" r in [0,P) is
 *    one selected pair; rows are ordered by expert (ascending), and by token
 *    (ascending) inside one expert.
 *  - All work is enqueued on the HIP stream given to evomoe_create; no call
 *    synchronises with the host except evomoe_num_pairs.  Outputs of one call
 *    may be used as inputs of the next without synchronisation.
 *  - Every call returns an evomoe_status.  Argument errors are detected on the
 *    host before anything is launched (no partial effects).  P > P_cap is
 *    data-dependent: evomoe_dispatch then raises a device-side flag, writes
 *    only rows < P_cap, and every later call clamps to P_cap (results are then
 *    meaningless but all accesses stay in bounds); evomoe_num_pairs reports
 *    EVOMOE_ECAPACITY.
 *  - Identical inputs give bit-identical outputs (no floating-point atomics).
 *  - Limits: 1 <= E <= 64; d and F multiples of 8 (bf16) or 4 (f32);
 *    T*E and P_cap below 2^31 (P_cap*max(d,F) may exceed 2^31: row bases are
 *    64-bit).  The bf16 expert FFN (forward and backward) additionally needs
 *    d >= 64, F >= 64, T below 2^24, and T*max(d,F)*2 and d*F*2 below 2^32 bytes
 *    (inside a tile its kernels add 32-bit byte offsets to a 64-bit base).
 */
#ifndef EVOMOE_H
#define EVOMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct evomoe_ctx evomoe_ctx;

typedef enum {
    EVOMOE_OK = 0,
    EVOMOE_EINVAL = -1,        /* null pointer, non-positive size, bad enum, misaligned pointer */
    EVOMOE_EUNSUPPORTED = -2,  /* valid request outside the limits above */
    EVOMOE_ECAPACITY = -3,     /* P exceeded P_cap (reported by evomoe_num_pairs) */
    EVOMOE_EWORKSPACE = -4,    /* workspace too small / null */
    EVOMOE_EHIP = -5,          /* a HIP runtime call failed */
    EVOMOE_ESTATIC = -6        /* evomoe_dispatch_static: the shape needs more than the library's static scratch */
} evomoe_status;

typedef enum { EVOMOE_F32 = 0, EVOMOE_BF16 = 1 } evomoe_dtype;
typedef enum { EVOMOE_RELU = 0, EVOMOE_GELU_ERF = 1 } evomoe_act;   /* Eq. ffn uses ReLU; the experiments GeLU = x*Phi(x) */

typedef struct {
    int32_t T, d, E, F;
    int32_t dtype;   /* evomoe_dtype */
    int32_t act;     /* evomoe_act   */
    int64_t P_cap;   /* rows available in every per-pair buffer; T*E never overflows */
} evomoe_shape;

/* Create / destroy a context bound to one HIP stream (hipStream_t passed as void*; NULL = default
 * stream) on the current device.  The context owns only small device scratch (per-block expert
 * histograms, a status word and, for a bf16 layer, W_g split into three bf16 planes); it may grow that scratch, with a device allocation, the first time a
 * larger T is seen.  Not thread-safe: one context per host thread/stream. */
evomoe_status evomoe_create(evomoe_ctx** ctx_out, void* hip_stream);
evomoe_status evomoe_destroy(evomoe_ctx* ctx);
const char*   evomoe_status_string(evomoe_status s);

/* Bytes of caller-provided device workspace that is enough for any single call below on this
 * shape (calls on one stream may share it).  Returns 0 for an invalid shape. */
size_t evomoe_workspace_bytes(const evomoe_shape* shape);

/* DTS gate forward (Stage 2: Eq. gumbel_softmax, Eq. adaptive_sparsity; Algorithm 2, threshold branch).
 *   in : x [T,d] elem; Wg [d,E] f32 (D x N as in the paper); bg [E] f32 or NULL;
 *        noise [T,E] f32 (pre-drawn Gumbel(0,1) samples zeta) or NULL for no noise;
 *        tau > 0; threshold c >= 0 (the test is strict: g' > c).
 *   out: gprime [T,E] f32 = g'; gate_w [T,E] f32 = g' where selected else 0, NOT renormalised (may be NULL);
 *        mask_bits [T] u64, bit i set <=> expert i selected for the token;
 *        counts [E] i32 = tokens selected per expert; k_per_token [T] i32 (may be NULL);
 *        block_hist [ceil(T/256), E] i32 (may be NULL): row b = tokens selected per expert among tokens
 *        256 b .. 256 b + 255, the table evomoe_dispatch starts from (handing it over saves that call a pass
 *        over mask_bits).
 * A token with no score above c keeps its arg-max expert (lowest index on ties), so 1 <= k_s <= E. */
evomoe_status evomoe_dts_gate(evomoe_ctx* ctx, const evomoe_shape* shape,
                              const void* x, const float* Wg, const float* bg, const float* noise,
                              float tau, float threshold,
                              float* gprime, float* gate_w, uint64_t* mask_bits,
                              int32_t* counts, int32_t* k_per_token, int32_t* block_hist);

/* Top-1 branch of the DTS gate (Algorithm 2, else-branch: iterations >= T_D; "switch to Top1" in the
 * temperature-scheduler study).  Same inputs and outputs as evomoe_dts_gate without a threshold: every
 * token selects its arg-max expert (lowest index on ties) with weight g' of that expert, not renormalised,
 * so k_s = 1 and P = T.  Every later step (dispatch ... gate backward) is the same call as for the
 * threshold branch. */
evomoe_status evomoe_dts_gate_top1(evomoe_ctx* ctx, const evomoe_shape* shape,
                                   const void* x, const float* Wg, const float* bg, const float* noise,
                                   float tau,
                                   float* gprime, float* gate_w, uint64_t* mask_bits,
                                   int32_t* counts, int32_t* k_per_token, int32_t* block_hist);

/* Balance loss (Eq. balance_loss):  L = alpha * N * sum_i (count_i / T^2) * sum_s g'_si,
 * and its gradient with respect to g'_si, which is the same for every token: coef_i = alpha * N * count_i / T^2
 * (the indicator count is a constant of the differentiation).
 *   in : gprime [T,E] f32, counts [E] i32 (both as written by the gate), alpha.
 *   out: loss [1] f32 (device), dgprime_coef [E] f32 (device; may be NULL).
 * Deterministic (fixed summation order). */
evomoe_status evomoe_balance_loss(evomoe_ctx* ctx, const evomoe_shape* shape,
                                  const float* gprime, const int32_t* counts, float alpha,
                                  float* loss, float* dgprime_coef);

/* Dispatch (Algorithm 1: the loop over id in id_s, turned into a permutation).  Stable counting
 * sort of the selected pairs: expert-major, token-ascending.
 *   in : mask_bits [T] (bits of experts >= E are ignored); scores [T,E] f32 (g' or gate_w: only selected entries
 *        are read); block_hist (last argument) [ceil(T/256), E] i32 as written by the gate for THIS mask_bits, or
 *        NULL (the call then counts the table itself; a table that does not match mask_bits gives wrong rows).
 *   out: expert_offsets [E+1] i32 (row range of expert i is [off[i], off[i+1]); off[E] = P);
 *        pair_token [P_cap] i32 (token of row r); pair_gate [P_cap] f32 (its weight G);
 *        tok_off [T+1] i32 and tok_rows [P_cap] i32: token s owns rows tok_rows[tok_off[s] .. tok_off[s+1])
 *        in ascending expert id; num_pairs [1] i64 = P (device).
 *        x_perm [P_cap,d] elem, optional (NULL = not materialised; needs x): x_perm[r,:] = x[pair_token[r],:]. */
evomoe_status evomoe_dispatch(evomoe_ctx* ctx, const evomoe_shape* shape,
                              const uint64_t* mask_bits, const float* scores,
                              int32_t* expert_offsets, int32_t* pair_token, float* pair_gate,
                              int32_t* tok_off, int32_t* tok_rows, int64_t* num_pairs,
                              const void* x, void* x_perm, const int32_t* block_hist);

/* evomoe_dispatch for callers that cannot allocate device memory at the moment of the call: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results as
 * evomoe_dispatch without a block_hist table; the per-256-token histograms it counts go into a table that is part
 * of the library image (256 KB on every GPU the library runs on, held until the process ends) instead of the
 * context's scratch, which evomoe_dispatch may have to grow with a device allocation.  This call never allocates
 * or frees.  Limit: ceil(T/256) * E <= 65536, else EVOMOE_ESTATIC and nothing is launched.  All calls on one GPU
 * share the one table, whatever their context or stream: calls that overlap in time on one GPU race (calls on
 * one stream do not overlap).  The table needs no clearing: every entry a call reads it has written before. */
evomoe_status evomoe_dispatch_static(evomoe_ctx* ctx, const evomoe_shape* shape,
                                     const uint64_t* mask_bits, const float* scores,
                                     int32_t* expert_offsets, int32_t* pair_token, float* pair_gate,
                                     int32_t* tok_off, int32_t* tok_rows, int64_t* num_pairs,
                                     const void* x, void* x_perm);

/* Expert FFNs forward over the ragged per-expert row ranges (Eq. ffn per expert e_i : R^D -> R^D).
 *   in : x [T,d] elem gathered through pair_token [P_cap], or, if pair_token == NULL, x is already
 *        the permuted [P_cap,d]; expert_offsets [E+1]; W1 [E,F,d] elem, b1 [E,F] f32 (NULL = 0),
 *        W2 [E,d,F] elem, b2 [E,d] f32 (NULL = 0).
 *   out: H [P_cap,F] elem = W1 x + b1 (pre-activation, kept for backward);
 *        A [P_cap,F] elem = act(H); O [P_cap,d] elem = W2 A + b2 = e_i(x_s). */
evomoe_status evomoe_expert_ffn(evomoe_ctx* ctx, const evomoe_shape* shape,
                                const void* x, const int32_t* pair_token, const int32_t* expert_offsets,
                                const void* W1, const float* b1, const void* W2, const float* b2,
                                void* H, void* A, void* O);

/* Combine (Eq. moe_weighted_sum_problem): y[s,:] = sum over the token's rows r, ascending expert,
 * of pair_gate[r] * O[r,:], accumulated in f32.   out: y [T,d] elem. */
evomoe_status evomoe_combine(evomoe_ctx* ctx, const evomoe_shape* shape,
                             const void* O, const float* pair_gate,
                             const int32_t* tok_off, const int32_t* tok_rows, void* y);

/* Backward of combine (the derivative of Eq. moe_weighted_sum_problem, y_s = sum_r G_r O_r, with respect to each
 * expert output and each weight; the paper derives no backward):
 *   dO[r,:] = pair_gate[r] * dy[pair_token[r],:];  dG_pairs[r] = <dy[pair_token[r],:], O[r,:]>.
 *   in : dy [T,d] elem, O, pair_gate, pair_token, expert_offsets (for P).  out: dO [P_cap,d] elem, dG_pairs [P_cap] f32. */
evomoe_status evomoe_combine_bwd(evomoe_ctx* ctx, const evomoe_shape* shape,
                                 const void* dy, const void* O, const float* pair_gate,
                                 const int32_t* pair_token, const int32_t* expert_offsets,
                                 void* dO, float* dG_pairs);

/* Backward of the expert FFNs (calculus on Eq. ffn; the paper derives none):
 *   db2_i = sum_rows dO;  dW2_i = dO_i^T A_i;  dA = dO_i W2_i;  dH = dA * act'(H);
 *   db1_i = sum_rows dH;  dW1_i = dH_i^T X_i;  dXp = dH W1_i.
 *   in : dO [P_cap,d], H, A [P_cap,F], x / pair_token as in the forward, expert_offsets, W1, W2;
 *        dy [T,d] elem and pair_gate [P_cap] f32, optional (both or neither; need pair_token): the inputs dO was
 *        made from, dO[r,:] = pair_gate[r] * dy[pair_token[r],:].  When given, a bf16 layer evaluates
 *        dA = pair_gate[r] * (dy[pair_token[r],:] W2_i) with the weight applied in float32, so that the bf16
 *        rounding of the stored dO stays out of dH, dXp, dW1 and db1 (dW2 and db2 are sums over dO itself).
 *   out: dW1 [E,F,d] elem, db1 [E,F] f32, dW2 [E,d,F] elem, db2 [E,d] f32 (each may be NULL to skip),
 *        dXp [P_cap,d] elem (gradient w.r.t. each row's input).
 *   accumulate != 0 adds the weight/bias gradients to the buffers' current contents.
 *   workspace: at least evomoe_workspace_bytes(shape) bytes (holds dH). */
evomoe_status evomoe_expert_ffn_bwd(evomoe_ctx* ctx, const evomoe_shape* shape,
                                    const void* dO, const void* H, const void* A,
                                    const void* x, const int32_t* pair_token, const int32_t* expert_offsets,
                                    const void* W1, const void* W2,
                                    const void* dy, const float* pair_gate,
                                    void* dW1, float* db1, void* dW2, float* db2, void* dXp,
                                    int accumulate, void* workspace, size_t workspace_bytes);

/* Backward of dispatch (Algorithm 1's loop over id in id_s hands x_s to each of the token's experts, so the
 * token's input gradient is the sum over them): dx[s,:] = sum of dXp over the token's rows (ascending expert,
 * f32 accumulate).
 *   out: dx [T,d] elem (overwritten). */
evomoe_status evomoe_dispatch_bwd(evomoe_ctx* ctx, const evomoe_shape* shape,
                                  const void* dXp, const int32_t* tok_off, const int32_t* tok_rows, void* dx);

/* Backward of the DTS gate: the derivative of Eq. gumbel_softmax (temperature softmax of x W_g + b_g + zeta)
 * followed by Eq. adaptive_sparsity, whose 0/1 selection is treated as a constant:
 *   dG_si = dG_pairs at the token's selected experts, 0 elsewhere;
 *   dz_sj = (g'_sj / tau) * (dG_sj - sum_i dG_si g'_si);  dWg = x^T dz;  dbg = sum_s dz_s;  dx_s += W_g dz_s.
 * Unselected experts' columns of W_g receive gradient through the softmax normaliser.
 *   in : dG_pairs [P_cap] f32, tok_off, tok_rows, gprime [T,E], mask_bits [T], tau, x [T,d] elem, Wg [d,E].
 *   out: dWg [d,E] f32, dbg [E] f32 (may be NULL), both overwritten; dx [T,d] elem is ACCUMULATED INTO
 *        (pass the output of evomoe_dispatch_bwd to obtain the full input gradient).
 *   workspace: at least evomoe_workspace_bytes(shape) bytes. */
evomoe_status evomoe_dts_gate_bwd(evomoe_ctx* ctx, const evomoe_shape* shape,
                                  const float* dG_pairs, const int32_t* tok_off, const int32_t* tok_rows,
                                  const float* gprime, const uint64_t* mask_bits, float tau,
                                  const void* x, const float* Wg,
                                  float* dWg, float* dbg, void* dx,
                                  void* workspace, size_t workspace_bytes);

/* evomoe_dts_gate_bwd with one more gradient flowing into g': dgprime_coef [E] f32 (as written by
 * evomoe_balance_loss), scaled by loss_scale, is added to dG_si for EVERY (s, i), selected or not, before the
 * softmax backward.  dgprime_coef == NULL is evomoe_dts_gate_bwd. */
evomoe_status evomoe_dts_gate_bwd_balance(evomoe_ctx* ctx, const evomoe_shape* shape,
                                          const float* dG_pairs, const int32_t* tok_off, const int32_t* tok_rows,
                                          const float* gprime, const uint64_t* mask_bits, float tau,
                                          const void* x, const float* Wg,
                                          const float* dgprime_coef, float loss_scale,
                                          float* dWg, float* dbg, void* dx,
                                          void* workspace, size_t workspace_bytes);

/* Backward of the expert FFNs that keeps no activations between forward and backward (the single-GPU
 * counterpart of the paper's MoE-aware recomputation, Implementation section): H and A are recomputed from x
 * by the forward's first GEMM into the workspace, then the backward proceeds as evomoe_expert_ffn_bwd.
 * Costs 14*d*F instead of 12*d*F flop per pair over forward + backward and saves 2*P_cap*F elements of
 * resident activations.  Arguments as evomoe_expert_ffn_bwd without H and A, plus b1 (dy and pair_gate optional,
 * as there).
 *   workspace: at least evomoe_workspace_bytes_recompute(shape) bytes. */
size_t evomoe_workspace_bytes_recompute(const evomoe_shape* shape);
evomoe_status evomoe_expert_ffn_bwd_recompute(evomoe_ctx* ctx, const evomoe_shape* shape,
                                              const void* dO,
                                              const void* x, const int32_t* pair_token, const int32_t* expert_offsets,
                                              const void* W1, const float* b1, const void* W2,
                                              const void* dy, const float* pair_gate,
                                              void* dW1, float* db1, void* dW2, float* db2, void* dXp,
                                              int accumulate, void* workspace, size_t workspace_bytes);

/* Training phase of an iteration (host only, no device work; Algorithm 1's loop bounds, Algorithm 2's T_D
 * switch, Sparsity Scheduler).  Iterations [0, T_S): stage 1 (one shared expert, this library is not
 * involved).  The next T_D iterations: threshold gate, tau going linearly from tau_hi to tau_lo with both end
 * points reached.  From T_S + T_D on: Top-1 gate at tau_lo. */
typedef struct {
    int32_t stage;   /* 1 = expert-diversify, 2 = gate-sparsify */
    int32_t top1;    /* stage 2: 0 = evomoe_dts_gate, 1 = evomoe_dts_gate_top1 */
    float tau;       /* stage 2 only (NaN in stage 1) */
} evomoe_phase;
evomoe_status evomoe_schedule(int64_t iteration, int64_t T_S, int64_t T_D, float tau_hi, float tau_lo,
                              evomoe_phase* phase_out);

/* Expert-diversify (Stage 1 "Expert-Diversify"; Algorithm 1, the loop e_i <- diversify(e, i)): spawns the E experts
 * of the layer from the one shared expert by setting a random part of its weights to 0, a different part for each
 * expert.  The paper gives neither the masked fraction nor the random source: mask_ratio in [0,1] is the probability
 * with which each weight of W1 and W2 is masked, independently; biases are copied unmasked.  The random numbers are
 * counter-based, so the result depends only on (seed, mask_ratio): weight number j (row-major) of tensor t (0 = W1,
 * 1 = W2) of expert i is masked when the top 24 bits of output number (t << 62 | i << 48 | j) of the SplitMix64
 * sequence seeded with `seed` are below floor(mask_ratio * 2^24).
 *   in : W1_shared [F,d] elem, b1_shared [F] f32 (may be NULL), W2_shared [d,F] elem, b2_shared [d] f32 (may be NULL).
 *   out: W1 [E,F,d] elem, b1 [E,F] f32 (NULL iff b1_shared is), W2 [E,d,F] elem, b2 [E,d] f32 (NULL iff b2_shared is).
 * T and P_cap of the shape are not used. */
evomoe_status evomoe_diversify(evomoe_ctx* ctx, const evomoe_shape* shape,
                               const void* W1_shared, const float* b1_shared,
                               const void* W2_shared, const float* b2_shared,
                               uint64_t seed, float mask_ratio,
                               void* W1, float* b1, void* W2, float* b2);

/* Copies P to the host and reports a pending capacity overflow.  The only synchronising call. */
evomoe_status evomoe_num_pairs(evomoe_ctx* ctx, const int64_t* num_pairs, int64_t* num_pairs_host);

/* Host only, no device work.  Announces the number of selected pairs the next calls will see (for instance the
 * previous iteration's evomoe_num_pairs: the Sparsity Scheduler changes P slowly).  The expert-FFN calls pick
 * their tile shapes for that many rows instead of for P_cap rows; results do not depend on it, buffers and
 * launch grids stay sized for P_cap.  expected_pairs <= 0 withdraws the announcement. */
evomoe_status evomoe_hint_pairs(evomoe_ctx* ctx, int64_t expected_pairs);

/* ---- measurement aid (not part of the layer) ----------------------------------------------------
 * Times kernels with HIP events recorded around their launches on the context's own stream.
 * evomoe_profile_select(ctx, id): id = one evomoe_kernel_id -> only that kernel is bracketed;
 * EVOMOE_K_ALL -> every kernel; EVOMOE_K_NONE -> off (default).  Events accumulate until read.
 * evomoe_profile_read synchronises the stream, writes per-kernel totals (milliseconds) and launch
 * counts into host arrays of EVOMOE_K_COUNT entries, and clears the record. */
typedef enum {
    EVOMOE_K_GATE = 0, EVOMOE_K_DISPATCH_HIST, EVOMOE_K_DISPATCH_SCATTER, EVOMOE_K_FFN_GEMM1,
    EVOMOE_K_FFN_GEMM2, EVOMOE_K_COMBINE, EVOMOE_K_COMBINE_BWD, EVOMOE_K_FFN_BWD_DH,
    EVOMOE_K_FFN_BWD_DX, EVOMOE_K_FFN_BWD_DW2, EVOMOE_K_FFN_BWD_DW1, EVOMOE_K_FFN_BWD_DB,
    EVOMOE_K_DISPATCH_BWD, EVOMOE_K_GATE_BWD_DZ, EVOMOE_K_GATE_BWD_MAIN, EVOMOE_K_GATE_BWD_REDUCE,
    EVOMOE_K_BALANCE_LOSS, EVOMOE_K_DIVERSIFY,
    EVOMOE_K_COUNT, EVOMOE_K_ALL = -2, EVOMOE_K_NONE = -1
} evomoe_kernel_id;
evomoe_status evomoe_profile_select(evomoe_ctx* ctx, int kernel_id);
evomoe_status evomoe_profile_read(evomoe_ctx* ctx, double* total_ms_host, int64_t* launches_host);

#ifdef __cplusplus
}
#endif
#endif /* EVOMOE_H */
