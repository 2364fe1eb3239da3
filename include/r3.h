/*
 * r3.h - C ABI of the replayed-routing MoE layer for AMD MI355X (gfx950).
 *
 * The calls follow Section 4.1 ("Implementation") of "Stabilizing MoE
 * Reinforcement Learning by Aligning Training and Inference Routers"
 * (arxiv 2510.11370): the MoE layer of the training pass is run with the
 * expert mask recorded at inference, while the softmax is still taken over the
 * training logits so that the router keeps its gradient.
 *
 * Notation: T tokens, d hidden size, E experts (the paper's M), K selected
 * experts per token, F width of one SwiGLU expert.  A slot is one (token t, j)
 * pair with id t*K + j; there are T*K slots.  "row" is a slot's position after
 * the slots are sorted by expert.
 *
 * Conventions for every call
 *  - All data pointers are DEVICE pointers owned by the caller.  The calls
 *    declared in this header allocate nothing, free nothing and keep no state
 *    between calls (the one exception is spelled out at r3_permute_static: a
 *    fixed scratch array and its cached address).  Scratch comes from a caller
 *    workspace of at least r3_workspace_bytes(desc, op) bytes, 256-byte
 *    aligned.  (The measurement aids of r3_profile.h are not part of the
 *    method and do keep state: event pools and an on/off flag.)
 *  - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work
 *    and return; there is no hidden synchronisation.
 *  - Matrices are row-major and dense.  Activations and weights have the dtype
 *    desc->act (bf16 or f32); gates, logits and weight gradients are f32;
 *    counts, offsets and permutations are int32.
 *  - The return value is an r3_status.  Errors the host can see (NULL pointer,
 *    bad sizes, misaligned pointer, small workspace) are returned before
 *    anything is launched.  Errors only the device can see (an expert id >= E,
 *    a duplicate id inside a token, a non-finite logit) OR bits into the
 *    optional device word `status_word` (R3_DATA_*); the affected token's
 *    outputs are then unspecified but no access goes out of bounds.
 *  - Every result is deterministic: the same inputs give the same bits.
 */
#ifndef R3_H
#define R3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum r3_status {
    R3_OK = 0,
    R3_ERR_INVALID_ARG = 1, /* NULL pointer, size <= 0, K > E, misaligned pointer  */
    R3_ERR_UNSUPPORTED = 2, /* index dtype too narrow for E, E or K above a kernel limit */
    R3_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than r3_workspace_bytes   */
    R3_ERR_HIP = 4          /* a launch failed                                     */
} r3_status;

enum { R3_BF16 = 0, R3_F32 = 1 };     /* desc->act   */
enum { R3_IDX_U8 = 0, R3_IDX_U16 = 1 }; /* desc->idx   */

/* bits of the device status word */
enum { R3_DATA_IDX_RANGE = 1, R3_DATA_IDX_DUP = 2, R3_DATA_NONFINITE = 4, R3_DATA_CACHE_ADDR = 8 };

typedef enum r3_op {
    R3_OP_REPLAY_GATE = 0,
    R3_OP_PERMUTE = 1,
    R3_OP_GROUPED_FFN = 2,
    R3_OP_BACKWARD = 3,
    R3_OP_FORWARD = 4       /* r3_moe_forward */
} r3_op;

enum { R3_FLAG_GATED_H = 1 };         /* desc->flags */

typedef struct r3_layer_desc {
    int32_t T, d, E, K, F;
    int32_t act;              /* R3_BF16 or R3_F32                                  */
    int32_t idx;              /* R3_IDX_U8 (E <= 256) or R3_IDX_U16 (E <= 65536)     */
    int32_t flags;            /* 0, or R3_FLAG_GATED_H for r3_moe_backward after
                                 r3_moe_forward (see there)                          */
    int64_t idx_token_stride; /* elements between two tokens' records; 0 means K.
                                 K gives a layer-major record [L][T][K]; L*K a
                                 token-major one [T][L][K] (Section 4.2: the
                                 inference side appends per token).               */
} r3_layer_desc;

/* Limits of this build: E <= 4096, K <= 64, K <= E. */

/* Bytes of workspace `op` needs for this layer (0 is possible). */
size_t r3_workspace_bytes(const r3_layer_desc *desc, r3_op op);

/* Human-readable build string. */
const char *r3_version(void);

/*
 * TopKMask(s, K) of Section 4.1 (second equation; used on the inference logits
 * to make the record I_infer).  For each of the T rows of `logits` ([T, ld]
 * f32, first E columns used) write the ids of the K largest entries to
 * `idx_out` ([T] records of K ids, stride desc->idx_token_stride), ascending by
 * id.  Ties go to the lower id; NaN ranks below every number; -0 equals +0.
 * A NaN or infinity sets R3_DATA_NONFINITE.
 */
int r3_record_topk(const r3_layer_desc *desc, const float *logits, int64_t ld,
                   void *idx_out, int32_t *status_word, void *stream);

/*
 * Router logits and replay gate of Section 4.1: s = x W_r (+ bias), then
 * g[t,j] = exp(s[t,idx[t,j]]) / sum_i exp(s[t,idx[t,i]]) over the K recorded
 * experts (replay-gate equation).  x [T,d] act, W_r [d,E] act, bias [E] f32 or
 * NULL, idx the record, gates [T,K] f32 aligned with idx.  Logits are
 * accumulated and kept in f32.  Optional outputs: logits_out [T,E] f32;
 * agree_out int64[2] which is INCREMENTED by {tokens whose own top-K set equals
 * the recorded set, total experts the two sets share} (Section 3.2, router
 * level; zero it before the first call).
 */
int r3_replay_gate(const r3_layer_desc *desc, const void *x, const void *W_r,
                   const float *bias, const void *idx, float *gates,
                   float *logits_out, int64_t *agree_out, int32_t *status_word,
                   void *ws, size_t ws_bytes, void *stream);

/*
 * Dispatch implied by the replay-output equation of Section 4.1: sort the T*K
 * slots by recorded expert, stably (ascending slot id inside an expert).
 * counts [E], offsets [E+1] (exclusive prefix sum), inv_perm [T*K] slot -> row,
 * perm [T*K] row -> slot, Xp [T*K,d] act with Xp[row] = x[perm[row] / K]
 * (Xp may be NULL to skip the row gather).  Sets R3_DATA_IDX_RANGE /
 * R3_DATA_IDX_DUP for a bad record.
 */
int r3_permute(const r3_layer_desc *desc, const void *x, const void *idx,
               int32_t *counts, int32_t *offsets, int32_t *inv_perm, int32_t *perm,
               void *Xp, int32_t *status_word, void *ws, size_t ws_bytes,
               void *stream);

/*
 * r3_permute for callers that cannot allocate or carry a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and status bits as r3_permute, without `ws`: the
 * scratch (per-chunk expert histograms and their running sums) is a fixed
 * array of R3_STATIC_SCRATCH_BYTES inside the library's device code, one copy
 * per GPU, held until the process ends; nothing is allocated or freed, by
 * this call or by anything it uses.  Its device address is looked up on the
 * first call on each device (with that device current) and kept.
 * Returns R3_ERR_UNSUPPORTED when r3_workspace_bytes(desc, R3_OP_PERMUTE)
 * exceeds R3_STATIC_SCRATCH_BYTES (that is (T*K/1024 rounded up, at most 512)
 * * E * 8 bytes: E <= 1024 always fits), R3_ERR_HIP when the address lookup
 * fails.  All calls on one GPU share the one array, on every stream: two calls
 * that overlap in time on a GPU race; calls ordered by a stream or an event
 * are fine (every word that is read is written first by the same call).
 */
#define R3_STATIC_SCRATCH_BYTES (4u << 20)
int r3_permute_static(const r3_layer_desc *desc, const void *x, const void *idx,
                      int32_t *counts, int32_t *offsets, int32_t *inv_perm, int32_t *perm,
                      void *Xp, int32_t *status_word, void *stream);

/*
 * The expert networks E_i of the replay-output equation, as bias-free SwiGLU:
 * for expert e and its rows r in [offsets[e], offsets[e+1]):
 *   A = Xp W_gate[e], B = Xp W_up[e], H = silu(A) * B, Yp = H W_down[e].
 * Xp [T*K,d]; W_gate, W_up [E,d,F]; W_down [E,F,d]; Yp [T*K,d]; H [T*K,F]
 * (required: it is the second GEMM's input and the backward's saved value).
 * FA_save, FB_save [T*K,F] or both NULL (forward only): what the backward
 * needs of the pre-activations, as the two factors its SwiGLU step multiplies
 * with: FA = B * silu'(A) (so that dA = dh * FA) and FB = silu(A) (dB = dh * FB),
 * silu'(a) = s (1 + a (1 - s)), s = sigmoid(a).  A and B themselves are not
 * stored.  All act dtype; f32 accumulation; `offsets` is read on the device.
 * Xp may be NULL when x [T,d] and perm [T*K] (from r3_permute) are given: row
 * r is then read as x[perm[r] / K] inside the first contraction's tile loads
 * and no gathered copy of the tokens is needed (r3_permute may be called with
 * Xp = NULL as well); needs T*d*sizeof(act) < 2^31.  x and perm are ignored
 * when Xp is given.
 */
int r3_grouped_ffn(const r3_layer_desc *desc, const void *Xp, const void *x, const int32_t *perm,
                   const int32_t *offsets, const void *W_gate, const void *W_up, const void *W_down,
                   void *Yp, void *H, void *FA_save, void *FB_save, void *ws,
                   size_t ws_bytes, void *stream);

/*
 * Replay output of Section 4.1: y[t] = sum_j gates[t,j] * Yp[inv_perm[t*K+j]],
 * j ascending, f32 accumulation, one rounding to act.  y [T,d].
 */
int r3_combine(const r3_layer_desc *desc, const void *Yp, const float *gates,
               const int32_t *inv_perm, void *y, void *stream);

/*
 * The replayed forward in one call (Section 4.1: router logits, replay gate,
 * and the replay-output equation y = sum_i g_i E_i(x) over the recorded
 * experts).  Same results as r3_replay_gate, r3_permute (without the gathered
 * copy), r3_grouped_ffn and r3_combine in a row, to the same tolerance, with
 * the gate folded into the expert network: the first contraction's epilogue
 * stores g_r * silu(A) * B for row r (g_r the gate of the row's slot), so the
 * down projection yields the gated rows g_i E_i(x) and the combination is a
 * plain sum of each token's K rows (j ascending, f32, one rounding).  The
 * gradient of W_down then finds its row operand ready, and the backward
 * neither forms g * dy per slot nor reads the expert outputs.
 * Outputs: y [T,d]; gates [T,K]; counts, offsets, inv_perm, perm as
 * r3_permute; H [T*K,F] = g * silu(A) * B (NOT r3_grouped_ffn's H); FA_save,
 * FB_save [T*K,F] as r3_grouped_ffn (both NULL: forward only); Yp [T*K,d] =
 * the gated rows.  logits_out, agree_out, status_word: as r3_replay_gate and
 * r3_permute.  ws: r3_workspace_bytes(desc, R3_OP_FORWARD).  desc->flags is
 * ignored.  To differentiate, pass these tensors to r3_moe_backward with
 * desc->flags = R3_FLAG_GATED_H.  Needs T*d*sizeof(act) < 2^31.
 */
int r3_moe_forward(const r3_layer_desc *desc, const void *x, const void *W_r, const float *bias,
                   const void *idx, const void *W_gate, const void *W_up, const void *W_down,
                   void *y, float *gates, int32_t *counts, int32_t *offsets, int32_t *inv_perm,
                   int32_t *perm, void *Yp, void *H, void *FA_save, void *FB_save,
                   float *logits_out, int64_t *agree_out, int32_t *status_word, void *ws,
                   size_t ws_bytes, void *stream);

/*
 * Backward of the replayed layer (Section 4.1, purpose (b): the gradient still
 * reaches the router logits through the softmax; the recorded mask is a
 * constant).  Given dy [T,d] act and the forward's tensors (FA, FB, H as
 * r3_grouped_ffn saved them), writes the gradient of sum(dy*y):  dx [T,d] act;
 * dW_r [d,E], dW_gate, dW_up [E,d,F], dW_down [E,F,d] f32;  dbias [E] f32 or
 * NULL.  accumulate = 0 overwrites the weight gradients, 1 adds to them.
 * Experts outside a token's recorded set get exactly zero router gradient from
 * that token.
 * bf16 shapes the MFMA kernels tile (d and F multiples of 256): perm is
 * required and T*d*sizeof(act) < 2^31 (else R3_ERR_UNSUPPORTED).  The expert
 * gradients read the rows of dy (and of x when Xp is NULL) through perm inside
 * their tile loads, and the softmax backward takes its dot products
 * <dy_t, o_j> from the down projection's gradient GEMM (<dy, H W_down> =
 * <dy W_down^T, H>), so no per-slot copy of dy is made and Yp is not read: Yp
 * and Xp may be NULL.  Other shapes and f32 run plain kernels, which need Xp
 * and Yp and do not read perm.
 * desc->flags = R3_FLAG_GATED_H: H and Yp are the gate-scaled tensors that
 * r3_moe_forward wrote (H = g silu(A) B, Yp = g o); perm is then required on
 * every path and Xp may be NULL on every path.
 */
int r3_moe_backward(const r3_layer_desc *desc, const void *dy, const void *x,
                    const void *W_r, const void *idx, const float *gates,
                    const int32_t *inv_perm, const int32_t *perm,
                    const int32_t *offsets, const void *Xp, const void *FA,
                    const void *FB, const void *H, const void *Yp, const void *W_gate,
                    const void *W_up, const void *W_down, void *dx, float *dW_r,
                    float *dW_gate, float *dW_up, float *dW_down, float *dbias,
                    int accumulate, void *ws, size_t ws_bytes, void *stream);

/*
 * Routing differences between two records of the same tokens (Section 3.2:
 * router-level, token-level and sequence-level comparison).  idx_a, idx_b:
 * device records of L layers, dtype desc->idx, K ids per router in any order;
 * the ids of token t in layer l start at element l*layer_stride +
 * t*token_stride (token_stride = desc->idx_token_stride, K if 0; layer-major
 * [L][T][K]: layer_stride = T*K; token-major [T][L][K]: token stride L*K,
 * layer_stride = K).  d = K - |A n B| is the number of differing choices of
 * one router.  Outputs (device): router_hist [K+1] int64, ADDED to (clear it
 * first): routers with d = 0..K;  token_choices [T] int32: d summed over the
 * layers;  token_routers [T] int32: layers with d > 0;  seq_mean [nseq] f64
 * or NULL: mean of token_routers over tokens seq_offsets[s]..seq_offsets[s+1]
 * (device int32 [nseq+1], ascending, within [0,T]).  Only T, K, E, idx and
 * idx_token_stride of desc are used.  All counts are exact.
 */
int r3_routing_diff(const r3_layer_desc *desc, int L, const void *idx_a, const void *idx_b,
                    int64_t layer_stride, const int32_t *seq_offsets, int nseq,
                    int64_t *router_hist, int32_t *token_choices, int32_t *token_routers,
                    double *seq_mean, void *stream);

/*
 * Policy discrepancy over n response tokens (Section 3.1): from the float32
 * log-probabilities of the sampled tokens under the training engine
 * (logp_train) and the inference engine (logp_infer), both device [n],
 *   *kl_out   = mean of r - 1 - log r,  r = exp(logp_train - logp_infer)
 *               (the k3 estimate of KL(pi_train || pi_infer), "KL Divergence
 *               Estimation"; evaluated in f64, fixed summation order),
 *   frac_out[i] = share of tokens with max(r, 1/r) > tau[i] (the extreme token
 *               distribution function F(tau)); the test |log r| > log tau is
 *               taken in float32 on the float32 difference, with
 *               log tau = float32(log(float64(tau))).
 * tau: HOST pointer, ntau <= 8 values >= 1 (read during the call); kl_out,
 * frac_out: device f64.  ws: device workspace of r3_policy_workspace_bytes().
 */
int r3_policy_discrepancy(int64_t n, const float *logp_train, const float *logp_infer, int ntau,
                          const float *tau, double *kl_out, double *frac_out, void *ws,
                          size_t ws_bytes, void *stream);
size_t r3_policy_workspace_bytes(void);

/*
 * Router-mask cache (Section 4.2: routing masks stored with the KV cache per
 * layer and token prefix, so that a prefix that hits the cache brings its masks
 * and is not prefilled again).  Masks live in `pages`, a device pool
 * [num_pages][P][L][K] of ids (idx_dtype R3_IDX_U8 / R3_IDX_U16): P tokens per
 * page, one token's L*K ids contiguous.  block_table: device int32
 * [nseq][max_blocks]; entry b of sequence s is the page that holds its tokens
 * b*P .. b*P+P-1 (negative: none).  A prefix shared by several sequences is the
 * same page ids in their rows; the library never allocates or frees pages.
 *
 * r3_mask_cache_append: ids of n new tokens (device; element (l, i, k) at
 * idx_new[l*layer_stride + i*token_stride + k], so both [n][L][K] and the
 * [L][n][K] that L calls of r3_record_topk leave are accepted) go to the slot of
 * token position[i] (0-based) of sequence seq_id[i] (device int32 [n]).  Two
 * entries that name the same slot race.
 *
 * r3_mask_cache_gather: the layer-major record out[L][T][K] of a packed batch:
 * sequence s owns tokens seq_start[s] .. seq_start[s+1]-1 (device int32
 * [nseq+1], ascending from 0 to T) and its j-th token is read from page
 * block_table[s][j / P], slot j % P.  The result is what r3_replay_gate,
 * r3_permute and r3_moe_backward take as idx, layer by layer.
 *
 * A token whose sequence, position or page is out of range is skipped by
 * append and zero-filled by gather, and R3_DATA_CACHE_ADDR is set in
 * *status_word (device, may be NULL); nothing is accessed out of bounds.
 * Pure copies: results are bit-exact.  pages, idx_new, out: aligned to the id
 * size.  n = 0 / T = 0 are no-ops.
 */
int r3_mask_cache_append(int idx_dtype, int L, int K, int P, void *pages, int64_t num_pages,
                         const int32_t *block_table, int nseq, int max_blocks, int64_t n,
                         const int32_t *seq_id, const int32_t *position, const void *idx_new,
                         int64_t layer_stride, int64_t token_stride, int32_t *status_word,
                         void *stream);
int r3_mask_cache_gather(int idx_dtype, int L, int K, int P, const void *pages, int64_t num_pages,
                         const int32_t *block_table, int nseq, int max_blocks,
                         const int32_t *seq_start, int64_t T, void *out, int32_t *status_word,
                         void *stream);

#ifdef __cplusplus
}
#endif
#endif /* R3_H */
