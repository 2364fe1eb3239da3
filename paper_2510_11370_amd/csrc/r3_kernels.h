// Internal launch interface between the C ABI (r3_api.hip) and the kernel files.
#pragma once
#include "r3_common.h"

namespace r3 {

// Optional per-kernel timing with HIP events on the launch stream (off by default).
// A ProfScope brackets one kernel launch; r3_profile_read() sums what was recorded.
enum ProfTag {
    PROF_RECORD = 0, PROF_LOGITS, PROF_GATE, PROF_PERMUTE_INDEX, PROF_GATHER_ROWS, PROF_FFN1, PROF_FFN2,
    PROF_COMBINE, PROF_GATE_BWD, PROF_DWR, PROF_DH, PROF_WGRAD, PROF_DXP, PROF_DX_FINISH, PROF_WGRAD_PAIR,
    PROF_ROUTING_DIFF, PROF_POLICY, PROF_CACHE_APPEND, PROF_CACHE_GATHER, PROF_AGREEMENT, PROF_NTAGS
};
struct ProfScope {
    int tag, slot;
    hipStream_t s;
    ProfScope(int tag, hipStream_t s);
    ~ProfScope();
};

// r3_route.hip
hipError_t launch_record_topk(int T, int E, int K, const float *logits, int64_t ld, void *idx,
                              int idx_dtype, int64_t stride, int32_t *status, hipStream_t s);
hipError_t launch_gate(int T, int E, int K, const float *logits, const void *idx, int idx_dtype,
                       int64_t stride, float *gates, int32_t *status, hipStream_t s);
hipError_t launch_agreement(int T, int E, int K, const float *logits, const void *idx, int idx_dtype,
                            int64_t stride, int64_t *agree, hipStream_t s);
size_t permute_ws_bytes(int T, int E, int K);
hipError_t launch_permute(int T, int d, int E, int K, int elem_bytes, const void *x, const void *idx,
                          int idx_dtype, int64_t stride, int32_t *counts, int32_t *offsets,
                          int32_t *inv_perm, int32_t *perm, void *Xp, int32_t *status, void *ws,
                          hipStream_t s);
hipError_t launch_combine(int T, int d, int K, int act, const void *Yp, const float *gates,
                          const int32_t *inv_perm, void *y, hipStream_t s);
// gated != 0: Yp holds gate-scaled rows (g o), so <dy, Yp_j> is already g_j dg_j
hipError_t launch_gate_backward(int T, int d, int E, int K, int act, const void *dy, const void *Yp,
                                const float *gates, const int32_t *inv_perm, const void *idx,
                                int idx_dtype, int64_t stride, void *dYp, float *dz, void *ds_dense,
                                int gated, hipStream_t s);
// masked-softmax backward from the row parts written by the expert-gradient GEMM:
// w_j = sum_p wpart[row_j][p] (= g_j dg_j), dz_j = w_j - g_j sum_i w_i; writes dz [T,K] and the dense
// bf16 ds [T,2E] (hi | lo halves)
hipError_t launch_gate_backward_parts(int T, int E, int K, int nparts, const float *wpart, const float *gates,
                                      const int32_t *inv_perm, const void *idx, int idx_dtype, int64_t stride,
                                      float *dz, void *ds_dense, hipStream_t s);
hipError_t launch_dx_finish(int T, int d, int E, int K, int act, const void *dXp, const void *WrT,
                            const float *dz, const int32_t *inv_perm, const void *idx, int idx_dtype,
                            int64_t stride, void *dx, hipStream_t s);
hipError_t launch_transpose(int R, int C, int act, const void *in, void *out, hipStream_t s);
hipError_t launch_colsum(int T, int E, int act, const void *ds, float *out, int accumulate, hipStream_t s);

// r3_diag.hip
size_t policy_ws_bytes();
int policy_max_tau();
hipError_t launch_routing_diff(int T, int K, int L, const void *a, const void *b, int idx_dtype, int64_t token_stride,
                               int64_t layer_stride, const int32_t *seq_offsets, int nseq, int64_t *router_hist,
                               int32_t *token_choices, int32_t *token_routers, double *seq_mean, hipStream_t s);
hipError_t launch_policy_discrepancy(int64_t n, const float *lt, const float *li, int ntau, const float *tau_host,
                                     double *kl, double *frac, void *ws, hipStream_t s);

// r3_cache.hip
hipError_t launch_cache_append(int idx_bytes, int L, int K, int P, void *pages, int64_t num_pages,
                               const int32_t *block_table, int nseq, int max_blocks, int64_t n,
                               const int32_t *seq_id, const int32_t *position, const void *idx_new,
                               int64_t layer_stride, int64_t token_stride, int32_t *status, hipStream_t s);
hipError_t launch_cache_gather(int idx_bytes, int L, int K, int P, const void *pages, int64_t num_pages,
                               const int32_t *block_table, int nseq, int max_blocks, const int32_t *seq_start,
                               int T, void *out, int32_t *status, hipStream_t s);

// r3_simt.hip
hipError_t simt_router_logits(int T, int d, int E, int act, const void *x, const void *Wr, const float *bias,
                              float *logits, hipStream_t s);
// perm != NULL: `Xp` is x [T,d] and row r of the grouped operand is x[perm[r] / K] (no gathered copy)
// grow != NULL: H is stored scaled by the row's gate (grow [S] f32)
hipError_t simt_ffn1(int S, int d, int E, int F, int act, const void *Xp, const int32_t *perm, int K,
                     const int32_t *offsets, const void *Wg, const void *Wu, void *H, void *A, void *B,
                     const float *grow, hipStream_t s);
hipError_t simt_ffn2(int S, int d, int E, int F, int act, const void *H, const int32_t *offsets, const void *Wd,
                     void *Yp, hipStream_t s);
hipError_t simt_dh(int S, int d, int E, int F, int act, const void *dYp, const int32_t *offsets, const void *Wd,
                   const void *A, const void *B, void *dA, void *dB, hipStream_t s);
hipError_t simt_dxp(int S, int d, int E, int F, int act, const void *dA, const void *dB, const int32_t *offsets,
                    const void *Wg, const void *Wu, void *dXp, hipStream_t s);
// ptok / qtok != NULL: that operand is an un-permuted matrix and row r of the reduction is its row tok[r]
hipError_t simt_wgrad(int E, int NP, int NQ, int act, const void *P, const int32_t *ptok, const void *Q,
                      const int32_t *qtok, const int32_t *offsets, float *out, int accumulate, hipStream_t s);
hipError_t simt_dwr(int T, int d, int E, int act, const void *x, const void *ds, float *dWr, int accumulate,
                    hipStream_t s);

// r3_gemm.hip (bf16 MFMA)
bool mfma_ffn_supported(int d, int F);
bool mfma_router_supported(int d, int E);
size_t mfma_tiles_bytes(int64_t S, int E);
size_t mfma_dwr_ws_bytes(int T, int d, int E);
// split_rows > 0: experts with more rows than that are cut into parts of at most that many rows for the
// weight gradients (mfma_wgrad_split_rows picks it); 0: never; < 0: the pass has no
// weight gradients and the table gets no reduction segments at all
hipError_t mfma_build_tiles(int E, const int32_t *offsets, int32_t *tiles, int split_rows, hipStream_t s);
// the same launch also makes the row -> token list and the per-row gates (see mfma_row_tokens)
hipError_t mfma_build_tiles_and_row_tokens(int E, const int32_t *offsets, int32_t *tiles, int split_rows, int S, int K,
                                           const int32_t *perm, const float *gates, int32_t *tok, float *grow,
                                           hipStream_t s);
// 0 unless `part_bytes_available` holds the partial products of every slot a split may use
int mfma_wgrad_split_rows(int64_t S, int tiles_per_seg, size_t part_bytes_available, size_t bytes_per_slot);
// perm != NULL: `Xp` is x [T,d] (T*d*2 bytes readable) and the first contraction gathers its rows
// through perm in the tile loads
hipError_t mfma_ffn_forward(int64_t S, int d, int E, int F, const void *Xp, const int32_t *perm, int K, int T,
                            const int32_t *offsets, const int32_t *tiles, const void *Wg, const void *Wu,
                            const void *Wd, void *Yp, void *H, void *FA, void *FB, const float *grow,
                            hipStream_t s);
// u = dy Wd^T with the rows of dy read through tok (row r is dy[tok[r]], dy is [T,d]); writes dA = g u FA,
// dB = g u FB, Hg = g H and wpart [S, 2 F/256] f32, whose row sums are g <dy, o> (see rowgemm_kernel<1>).
// Hg == NULL: H already holds g H (the one-call forward wrote it so) and nothing is written for it
hipError_t mfma_ffn_dh(int64_t S, int d, int E, int F, const void *dy, const int32_t *tok, int T, const float *grow,
                       const int32_t *offsets, const int32_t *tiles, const void *Wd, const void *FA, const void *FB,
                       const void *H, void *dA, void *dB, void *Hg, float *wpart, hipStream_t s);
hipError_t mfma_ffn_dxp(int64_t S, int d, int E, int F, const void *dA, const void *dB, const int32_t *offsets,
                        const int32_t *tiles, const void *Wg, const void *Wu, void *dXp, hipStream_t s);
// `tiles` is the table mfma_build_tiles() filled in this call sequence; `launch` (2..7) picks the
// tile counters of this launch: 0 and 1 belong to the forward pair and to dh / dxp.
// out (+)= Qs^T Ps per expert.  tok != NULL: Ps is the un-permuted [nrows, NPd] matrix and row r of the
// reduction is its row tok[r] (nrows * NPd * 2 < 2^31).  The reduction segments come from the table (an
// expert's rows, or parts of them when the table was built with split_rows > 0: then `part` must hold
// the partial products, and a second launch adds them to the gradient in a fixed order)
hipError_t mfma_wgrad(int E, int NQd, int NPd, const void *Qs, const void *Ps, const int32_t *tok, int nrows,
                      const int32_t *tiles, int launch, float *out, float *part, int accumulate, hipStream_t s);
// out0 (+)= Qs^T P0 and out1 (+)= Qs^T P1 per expert in one pass over Qs.  tok != NULL: Qs is the
// un-permuted [nrows, NQd] matrix and row r of the reduction is its row tok[r] (a list made by
// mfma_row_tokens; nrows * NQd * 2 < 2^31)
// `part` (split tables only, else NULL): room for the partial products of both gradients, 2 x the slots of
// mfma_wgrad's
hipError_t mfma_wgrad_pair(int E, int NQd, int NPd, const void *Qs, const int32_t *tok, int nrows, const void *P0,
                           const void *P1, const int32_t *tiles, int launch, float *out0, float *out1, float *part,
                           int accumulate, hipStream_t s);
// tok[r] = perm[r] / K (r < S), padded; mfma_row_tokens_bytes(S) bytes.  gates != NULL: also
// grow[r] = gates[perm[r]] (f32 [S])
size_t mfma_row_tokens_bytes(int64_t S);   // (the kernel is plain: every path may use it)
hipError_t mfma_row_tokens(int S, int K, const int32_t *perm, const float *gates, int32_t *tok, float *grow,
                           hipStream_t s);
hipError_t mfma_router_logits(int T, int d, int E, const void *x, const void *Wr, const float *bias,
                              float *logits, hipStream_t s);
// logits + replay gate (+ agreement counts) in one launch; E = 128 (see gate_fused_kernel)
bool mfma_gate_fused_supported(int d, int E, int K, bool want_agreement);
hipError_t mfma_gate_fused(int T, int d, int E, int K, const void *x, const void *Wr, const float *bias,
                           const void *idx, int idx_dtype, int64_t stride, float *gates, float *logits_out,
                           int64_t *agree, int32_t *status, hipStream_t s);
hipError_t mfma_dwr(int T, int d, int E, const void *x, const void *ds, float *part, float *dWr, int accumulate,
                    hipStream_t s);

}  // namespace r3
