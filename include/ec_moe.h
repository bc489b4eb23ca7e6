/*
 * ec_moe.h -- C ABI of the expert-choice Mixture-of-Experts layer for AMD
 * Instinct MI355X (gfx950 / CDNA4).
 *
 * The layer follows "Mixture-of-Experts with Expert Choice Routing"
 * (arXiv 2202.09368), Sec. 3.2:
 *   Eq. 1  k = n*c/e                      bucket size of every expert
 *   Eq. 2  S = Softmax(X.Wg);  G, I = TopK(S^T, k)
 *   Eq. 3  X_in = P.X (P = Onehot(I));  X_e[i] = act(X_in[i].W1[i]).W2[i]
 *   Eq. 4  X_out[l,:] = sum_{i,j} P[i,j,l] G[i,j] X_e[i,j,:]
 * Notation is the paper's: n tokens, d model width, e experts, c capacity
 * factor, k tokens per expert, d_ff expert hidden width (the paper's d').
 *
 * General conventions (all entry points)
 *  - Every tensor pointer is a DEVICE pointer owned by the caller, dense,
 *    row-major, no strides, 16-byte aligned.  The library never allocates or
 *    frees device memory; scratch comes from the caller's workspace `ws`
 *    (device pointer, 256-byte aligned, at least ec_moe_workspace_bytes()).
 *  - Calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL =
 *    the default stream).  Nothing synchronises.  Outputs are fully
 *    overwritten; no output needs to be cleared beforehand.
 *  - Sizes are int64_t; token indices int32_t (n < 2^31); S and G are always
 *    float.  `dtype` (ec_dtype) is the storage type of X, Wg, W1, W2, X_in,
 *    X_e, X_out: EC_F32 or EC_BF16 (bf16 operands, fp32 accumulation).
 *  - With EC_BF16, d and d_ff must be multiples of 8 (16-byte rows).
 *  - Every function returns an ec_status.  Arguments are validated on the
 *    host before anything is launched; on error nothing has been enqueued.
 *    EC_ERR_HIP means a launch failed: ec_moe_last_hip_error() returns the
 *    hipError_t of the calling thread's last failure.
 *  - Inputs must be finite; NaN/Inf give unspecified routing.
 *  - Calls that share a workspace must be ordered on one stream.
 */
#ifndef EC_MOE_H
#define EC_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EC_OK = 0,
    EC_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, k outside [1,n], bad enum, misaligned */
    EC_ERR_WORKSPACE = -2,   /* workspace null or smaller than required */
    EC_ERR_HIP = -3,         /* a HIP call failed; see ec_moe_last_hip_error() */
    EC_ERR_UNSUPPORTED = -4  /* valid request outside what the kernels cover */
} ec_status;

/* EC_BF16_HILO: storage and interface exactly as EC_BF16; the two intermediates that EC_BF16 hands to a
 * matrix-core product as single bf16 numbers -- H = act(A) into the second product of Eq. 3, and dX_e = G dY into
 * dW2 -- are carried as high part + remainder (two bf16 numbers, 2^-17), and X_e goes into the sum of Eq. 4
 * unrounded.  Those two products do twice the work.  It is for callers who need every element of large outputs
 * within 2e-2 of an unrounded reference: with EC_BF16 a token's output row scales with its gate values while that
 * error measure is relative to the whole tensor, and the worst element of tens of millions reaches 2-3e-2.
 * Honoured by ec_moe_expert_ffn, every ec_moe_forward* entry point, ec_moe_backward(_timed) and
 * ec_moe_workspace_bytes (d and d_ff multiples of 64, else EC_ERR_UNSUPPORTED); the routing and data-movement
 * entry points, and layers with identity experts, treat it as EC_BF16. */
typedef enum { EC_F32 = 0, EC_BF16 = 1, EC_BF16_HILO = 2 } ec_dtype;
typedef enum { EC_ACT_RELU = 0, EC_ACT_GELU = 1 /* exact erf form */, EC_ACT_IDENTITY = 2 } ec_act;

/* Largest number of experts the routing kernels accept. */
#define EC_MOE_MAX_EXPERTS 1024

/* Host only.  Sec. 3.2, Eq. 1: *k = floor(n*c/e), evaluated in double.
 * EC_ERR_INVALID_ARG if n, e <= 0, c <= 0, k == NULL, or k would fall outside [1, n]. */
int ec_moe_capacity(int64_t n, int64_t e, double c, int64_t* k);

/* Host only.  Bytes of workspace sufficient for ANY entry point below at these
 * sizes (d_ff may be 0 for identity experts; with_backward != 0 adds what
 * ec_moe_backward needs).  Returns 0 for invalid sizes, and for EC_BF16_HILO with
 * an FFN whose widths that mode does not cover. */
size_t ec_moe_workspace_bytes(int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff,
                              int dtype, int with_backward);

/* Sec. 3.2, Eq. 2 (first line) and Sec. 3.4: token-to-expert affinity scores.
 *   Z = X.Wg with fp32 accumulation; S[l,:] = softmax over the e experts of
 *   Z[l,:] (max-subtracted, fp32).
 * X [n,d] and Wg [d,e] in `dtype`.  S [n,e] and St [e,n] (the transpose, the
 * layout ec_moe_topk_tokens reads) are float outputs; either may be NULL but
 * not both.  e <= EC_MOE_MAX_EXPERTS.  ws is not used (NULL, 0 allowed). */
int ec_moe_gate(const void* X, const void* Wg, float* S, float* St,
                int64_t n, int64_t d, int64_t e, int dtype,
                void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.2, Eq. 2 (second line): G, I = TopK(S^T, k).  For every expert i the k
 * largest scores over the n tokens.  St [e,n] float, all values >= 0 (softmax
 * output; negative or NaN values are outside the contract).
 * I [e,k] int32: token indices; G [e,k] float: G[i,j] = St[i, I[i,j]] bit for bit.
 * Of several equal scores at the k-th place the lower token indices are
 * admitted.  The paper leaves the order inside a bucket open; here a bucket
 * lists its tokens by ascending token index, so the result is unique.
 * 1 <= k <= n.  ws is not used (NULL, 0 allowed). */
int ec_moe_topk_tokens(const float* St, int64_t n, int64_t e, int64_t k,
                       float* G, int32_t* I, void* ws, size_t ws_bytes, void* stream);

/* Limitations section: expert choice inside groups of tokens, so that a selection never looks
 * outside its group (the remedy proposed there for autoregressive use and small batches).  The n
 * tokens are `groups` equal runs of consecutive tokens (n % groups == 0); every (expert, group)
 * pair takes the k_g best of its run, ties and order as in ec_moe_topk_tokens.  G, I [e, groups*k_g]:
 * an expert's bucket lists group 0's tokens, then group 1's, ...; I holds indices into the whole
 * batch, so the bucket as a whole is in ascending token order.  1 <= k_g <= n/groups.
 * EC_ERR_UNSUPPORTED unless groups == 1 or a run is a multiple of 4 and at most 65536 tokens.
 * ws is not used (NULL, 0 allowed). */
int ec_moe_topk_tokens_grouped(const float* St, int64_t n, int64_t e, int64_t groups, int64_t k_g,
                               float* G, int32_t* I, void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.2, Eq. 3 (first line), the "shuffle" stage of Sec. 3.4:
 * X_in[i,j,:] = X[I[i,j],:].  X [n,d], X_in [e,k,d] in `dtype`; a bit-exact
 * copy.  Every I[i,j] must lie in [0,n) (not checked on the device), or be -1: an empty row
 * (token-choice routing), which is filled with zeros. */
int ec_moe_dispatch(const void* X, const int32_t* I, void* Xin,
                    int64_t n, int64_t d, int64_t e, int64_t k, int dtype, void* stream);

/* Sec. 3.2, Eq. 3 (second line): X_e[i] = act(X_in[i].W1[i]).W2[i], no bias.
 * X_in [e,k,d], W1 [e,d,d_ff], W2 [e,d_ff,d] (the paper's W2[i]^T stored
 * untransposed), X_e [e,k,d], all in `dtype`.  EC_BF16: fp32 accumulation, the
 * hidden activations H = act(A) are rounded to bf16 between the two products,
 * X_e is rounded to bf16.  A_save / H_save: optional [e,k,d_ff] outputs in
 * `dtype` (pre-activation A = X_in.W1 and H), kept for ec_moe_backward; NULL to
 * skip.  act = EC_ACT_IDENTITY is a plain two-matrix product. */
int ec_moe_expert_ffn(const void* Xin, const void* W1, const void* W2, void* Xe,
                      void* A_save, void* H_save,
                      int64_t e, int64_t k, int64_t d, int64_t d_ff, int act, int dtype,
                      void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.2, Eq. 4, the "unshuffle" stage of Sec. 3.4:
 * X_out[l,:] = sum over the (i,j) with I[i,j] = l of G[i,j] * X_e[i,j,:], and 0
 * for tokens no expert selected.  Deterministic: a token's contributions are
 * added in ascending expert order in fp32 and rounded once to `dtype`; no
 * floating-point atomics.  A token may appear at most once per expert (true of
 * any TopK output) and every I[i,j] must lie in [0,n) or be -1 (empty row, skipped).
 * X_e [e,k,d], G [e,k], I [e,k], X_out [n,d].  e <= EC_MOE_MAX_EXPERTS. */
int ec_moe_combine(const void* Xe, const float* G, const int32_t* I, void* Xout,
                   int64_t n, int64_t d, int64_t e, int64_t k, int dtype,
                   void* ws, size_t ws_bytes, void* stream);

/* ec_moe_combine for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, arithmetic
 * and order of additions as ec_moe_combine (bit-identical X_out); the token-major index is built in
 * a static device array of EC_MOE_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held
 * until the process ends) instead of in `ws`.  Nothing is allocated or freed, no memset is enqueued
 * (the index is cleared by a fill kernel).
 * Limit: the index must fit the array -- e <= 16: 4*n*(1 + cap) bytes with cap = 4, 8 or 16 slots
 * (the smallest that holds e); e > 16: 4*n*ceil(e/32) + 4*(n+1) + 4*e*k + 4096 bytes, each part rounded up
 * to 256.  Larger problems return EC_ERR_UNSUPPORTED and enqueue nothing.
 * All calls on one GPU share the array, which keeps the previous call's contents: calls that overlap
 * on one GPU (different streams, or threads without ordering) race; order them on one stream.
 * The array's device address is looked up at the first call on a GPU: make that call outside a capture. */
#define EC_MOE_STATIC_SCRATCH_BYTES (8u << 20)
int ec_moe_combine_static(const void* Xe, const float* G, const int32_t* I, void* Xout,
                          int64_t n, int64_t d, int64_t e, int64_t k, int dtype, void* stream);

/* Sec. 3.2, Eq. 1-4 in one call on one stream: gate, TopK over tokens,
 * dispatch, expert FFN, combine.  k = floor(n*c/e) as in ec_moe_capacity.
 * W1 = W2 = NULL with act = EC_ACT_IDENTITY runs identity experts (routing
 * only: X_e = X_in); d_ff is then ignored.  The gather of Eq. 3 is fused where nobody asks for its
 * result: into the first expert product's tile loads, or, with identity experts, into the combine's
 * row reads (X_in is then never written; pass Xin_out or Xe_out to have it materialised).
 * Optional outputs, each NULL to skip: S_out [n,e], G_out [e,k], I_out [e,k]
 * (int32), Xin_out [e,k,d], A_out / H_out [e,k,d_ff], Xe_out [e,k,d] -- the
 * tensors ec_moe_backward consumes.  X_out [n,d] is required. */
int ec_moe_forward(const void* X, const void* Wg, const void* W1, const void* W2, double c,
                   void* Xout, float* S_out, float* G_out, int32_t* I_out,
                   void* Xin_out, void* A_out, void* H_out, void* Xe_out,
                   int64_t n, int64_t d, int64_t e, int64_t d_ff, int act, int dtype,
                   void* ws, size_t ws_bytes, void* stream);

/* ec_moe_forward with the TopK of Eq. 2 taken inside each of `groups` equal runs of tokens (see
 * ec_moe_topk_tokens_grouped): k_g = floor((n/groups)*c/e) per (expert, group), buckets of
 * k = groups*k_g rows.  Workspace and optional outputs as in ec_moe_forward with that k.
 * groups = 1 is ec_moe_forward. */
int ec_moe_forward_grouped(const void* X, const void* Wg, const void* W1, const void* W2, double c,
                           int64_t groups, void* Xout, float* S_out, float* G_out, int32_t* I_out,
                           void* Xin_out, void* A_out, void* H_out, void* Xe_out,
                           int64_t n, int64_t d, int64_t e, int64_t d_ff, int act, int dtype,
                           void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.1: conventional token-choice routing, the baseline the paper argues against.  Every token
 * independently takes its m best experts of S[l,:] (m = 1: Switch Transformer, m = 2: GShard;
 * Sec. 3.4), ties to the lower expert index.  An expert's buffer has `cap` rows; all first
 * choices are placed before any second choice, ascending token index inside a rank of choice;
 * a token that finds the buffer full is dropped there (the paper only says that an expert takes at
 * most a maximum number of tokens; the placement order is this library's reading).
 * S [n,e] float.  Outputs: I [e,cap] int32 token index or -1 for an empty row; G [e,cap] float
 * = S[I[i,j], i] bit for bit, 0 in empty rows; load [e] int32 (optional) = tokens that chose the
 * expert before dropping, so load/cap - 1 is the over-capacity ratio of Sec. 3.1.
 * ec_moe_dispatch and ec_moe_combine accept such I: an empty row gathers zeros and adds nothing.
 * 1 <= m <= min(e, 8), 1 <= cap <= n.  ws: at least 32*n bytes. */
int ec_moe_token_choice(const float* S, int64_t n, int64_t e, int64_t m, int64_t cap,
                        float* G, int32_t* I, int32_t* load, void* ws, size_t ws_bytes, void* stream);

/* The layer of Eq. 3-4 behind token-choice routing: gate (Eq. 2, first line), ec_moe_token_choice
 * with cap = floor(n*c/e) (Eq. 1: with c = m the buffers match expert choice at equal cost, the
 * comparison of Sec. 3.4), dispatch, expert FFN, combine with the raw scores as weights.
 * Optional outputs, NULL to skip: S_out [n,e], G_out / I_out [e,cap], load_out [e],
 * Xin_out / Xe_out [e,cap,d], A_out / H_out [e,cap,d_ff] -- with k = cap they are what
 * ec_moe_backward consumes.  Workspace: ec_moe_workspace_bytes with k = cap. */
int ec_moe_forward_token_choice(const void* X, const void* Wg, const void* W1, const void* W2,
                                double c, int64_t m, void* Xout, float* S_out, float* G_out,
                                int32_t* I_out, int32_t* load_out, void* Xin_out, void* A_out,
                                void* H_out, void* Xe_out,
                                int64_t n, int64_t d, int64_t e, int64_t d_ff, int act, int dtype,
                                void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.3: expert choice with at most b experts per token.  A [e,n] solves
 *   max <S^T, A> + lambda H(A),  rows sum to k, columns sum to at most b, 0 <= A <= 1
 * by Dykstra's algorithm over the three constraint sets (the paper: lambda = 0.001, at most 100
 * iterations), and the buckets become TopK(A, k).  The paper prints neither the projections nor a
 * stopping rule; this library's reading: KL projections (row scaling to k, column scaling by
 * min(1, b / column sum), clipping at 1) with Dykstra's correction terms for the two inequality
 * sets, in the log domain in float64, exactly `iters` sweeps (rows, columns, box).
 * St [e,n] float scores; A [e,n] float output (rounded once at the end).  b > 0, lambda > 0,
 * 0 <= iters <= 100000.  ws: ec_moe_capped_workspace_bytes(n, e).  2*iters + 2 launches. */
size_t ec_moe_capped_workspace_bytes(int64_t n, int64_t e);
int ec_moe_capped_assignment(const float* St, int64_t n, int64_t e, int64_t k, double b, double lambda,
                             int64_t iters, float* A, void* ws, size_t ws_bytes, void* stream);

/* ec_moe_forward with the routing of Sec. 3.3: I = indices of TopK(A, k) with A from
 * ec_moe_capped_assignment on the layer's own scores; the gate weights stay G[i,j] = S[I[i,j], i]
 * (the paper replaces only the indices).  Optional outputs, NULL to skip: S_out [n,e], G_out / I_out
 * [e,k], A_out [e,n], Xe_out [e,k,d].  ws: ec_moe_workspace_bytes(n,d,e,k,d_ff,dtype,0)
 * + ec_moe_capped_workspace_bytes(n,e) + 4*e*n rounded up to 256.  Forward only. */
int ec_moe_forward_capped(const void* X, const void* Wg, const void* W1, const void* W2, double c,
                          double b, double lambda, int64_t iters, void* Xout, float* S_out, float* G_out,
                          int32_t* I_out, float* A_out, void* Xe_out,
                          int64_t n, int64_t d, int64_t e, int64_t d_ff, int act, int dtype,
                          void* ws, size_t ws_bytes, void* stream);

/* Gradient of <dY, X_out> through Eq. 2-4 with the selection I held constant
 * and the gate values G differentiable (Sec. 3.4: the gating network is
 * trained through the top-k function).  Inputs: dY [n,d] and the forward's
 * X, Wg, W1, W2, S [n,e], G, I [e,k], X_in [e,k,d], A, H [e,k,d_ff], X_e [e,k,d].
 * Outputs: dX [n,d] in `dtype`; dWg [d,e], dW1 [e,d,d_ff], dW2 [e,d_ff,d] float.
 * ws must come from ec_moe_workspace_bytes(..., with_backward = 1).
 * The pass depends on the routing only through S, G, I and the saved bucket tensors, so it also
 * serves ec_moe_forward_grouped (k = groups * k_g) and the buffers of token-choice routing: an
 * empty row (I = -1, with G = 0 and zero rows in X_in, A, H, X_e as the forward leaves them) gets
 * and passes no gradient. */
int ec_moe_backward(const void* dY, const void* X, const void* Wg, const void* W1, const void* W2,
                    const float* S, const float* G, const int32_t* I,
                    const void* Xin, const void* A, const void* H, const void* Xe,
                    void* dX, float* dWg, float* dW1, float* dW2,
                    int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int act, int dtype,
                    void* ws, size_t ws_bytes, void* stream);

/* Measurement aid: ec_moe_backward with a HIP event recorded on `stream` before the first and after every
 * stage of the pass; the call then WAITS for the last event (the only entry point that synchronises) and
 * writes the stages' durations in milliseconds to stage_ms (HOST pointer, EC_MOE_BWD_STAGES floats).
 * Stages, in order (ec_moe_backward_stage_name(i), NULL outside 0..EC_MOE_BWD_STAGES-1): dX_e and dG rows of
 * Eq. 4; dW2 = H^T dX_e; dA = (dX_e W2^T) act'(A); dW1 = X_in^T dA; dX_in = dA W1^T; the token-major index;
 * the softmax derivative dZ; the two gate products (dWg = X^T dZ, dZ Wg^T); the scatter-add into dX.
 * Results and errors as ec_moe_backward.  Creates and destroys its events (host objects; no device memory). */
#define EC_MOE_BWD_STAGES 9
int ec_moe_backward_timed(const void* dY, const void* X, const void* Wg, const void* W1, const void* W2,
                          const float* S, const float* G, const int32_t* I,
                          const void* Xin, const void* A, const void* H, const void* Xe,
                          void* dX, float* dWg, float* dW1, float* dW2,
                          int64_t n, int64_t d, int64_t e, int64_t k, int64_t d_ff, int act, int dtype,
                          void* ws, size_t ws_bytes, void* stream, float* stage_ms);
const char* ec_moe_backward_stage_name(int stage);

/* hipError_t (as int) of the calling thread's most recent EC_ERR_HIP, else 0. */
int ec_moe_last_hip_error(void);

/* Static, human-readable name of an ec_status value. */
const char* ec_moe_status_string(int status);

/* Library version, "major.minor". */
const char* ec_moe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EC_MOE_H */
