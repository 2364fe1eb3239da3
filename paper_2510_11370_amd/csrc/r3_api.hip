// C ABI of the replayed MoE layer: argument checks, workspace carving and the
// launch sequence of each call.  See include/r3.h for the contract.
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "r3_kernels.h"

using namespace r3;

namespace {

struct Dims {
    int T, d, E, K, F, act, idx, flags;
    int64_t stride, S;
    int eb;  // bytes per activation element
};

int check_desc(const r3_layer_desc *D, Dims &m) {
    if (!D) return R3_ERR_INVALID_ARG;
    if (D->T <= 0 || D->d <= 0 || D->E <= 0 || D->K <= 0 || D->F <= 0 || D->K > D->E || (D->flags & ~R3_FLAG_GATED_H) != 0)
        return R3_ERR_INVALID_ARG;
    if (D->act != R3_BF16 && D->act != R3_F32) return R3_ERR_INVALID_ARG;
    if (D->idx != R3_IDX_U8 && D->idx != R3_IDX_U16) return R3_ERR_INVALID_ARG;
    if (D->idx_token_stride != 0 && D->idx_token_stride < D->K) return R3_ERR_INVALID_ARG;
    if ((D->idx == R3_IDX_U8 && D->E > 256) || D->E > kMaxE || D->K > kMaxK) return R3_ERR_UNSUPPORTED;
    if ((int64_t)D->T * D->K > 0x7fffffffLL / 2) return R3_ERR_UNSUPPORTED;
    m.T = D->T; m.d = D->d; m.E = D->E; m.K = D->K; m.F = D->F; m.act = D->act; m.idx = D->idx; m.flags = D->flags;
    m.stride = D->idx_token_stride ? D->idx_token_stride : D->K;
    m.S = (int64_t)D->T * D->K;
    m.eb = D->act == R3_BF16 ? 2 : 4;
    return R3_OK;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
bool force_simt() {
    const char *v = getenv("R3_FORCE_SIMT");
    return v && v[0] == '1';
}
bool use_mfma_ffn(const Dims &m) { return m.act == R3_BF16 && mfma_ffn_supported(m.d, m.F) && !force_simt(); }
bool use_mfma_router(const Dims &m) { return m.act == R3_BF16 && mfma_router_supported(m.d, m.E) && !force_simt(); }

struct BwdWs {
    size_t dXp, dz, ds, WrT, dA, dB, tiles, part, tok, Hg, grow, wpart, total;
};
int row_parts(const Dims &m) { return 2 * (m.F / 256); }   // partial dot products per row (MFMA path)
BwdWs bwd_layout(const Dims &m) {
    BwdWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    const bool mf = use_mfma_ffn(m);
    w.dXp = take((size_t)m.S * m.d * m.eb);  // the plain kernels keep g*dy here first
    w.dz = take((size_t)m.T * m.K * sizeof(float));
    w.ds = take((size_t)m.T * m.E * (m.act == R3_BF16 ? 2 : 1) * m.eb);  // bf16: (hi, lo) halves
    w.WrT = take((size_t)m.E * m.d * m.eb);
    w.dA = take((size_t)m.S * m.F * m.eb);
    w.dB = take((size_t)m.S * m.F * m.eb);
    w.tiles = take(mf ? mfma_tiles_bytes(m.S, m.E) : 0);
    w.part = take(use_mfma_router(m) ? mfma_dwr_ws_bytes(m.T, m.d, m.E) : 0);
    w.tok = take(mfma_row_tokens_bytes(m.S));                    // row -> token list
    w.Hg = take(mf ? (size_t)m.S * m.F * m.eb : 0);              // gate-scaled H rows
    w.grow = take(mf ? (size_t)m.S * sizeof(float) : 0);         // row -> gate list
    w.wpart = take(mf ? (size_t)m.S * row_parts(m) * sizeof(float) : 0);
    w.total = o;
    return w;
}

struct FwdWs {
    size_t gate, perm, ffn, tok, grow, total;
};
FwdWs fwd_layout(const Dims &m) {
    FwdWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes, 256); return at; };
    w.gate = take((size_t)m.T * m.E * sizeof(float));
    w.perm = take(permute_ws_bytes(m.T, m.E, m.K));
    w.ffn = take(use_mfma_ffn(m) ? mfma_tiles_bytes(m.S, m.E) : 0);
    w.tok = take(mfma_row_tokens_bytes(m.S));
    w.grow = take((size_t)m.S * sizeof(float));
    w.total = o;
    return w;
}

int hip_rc(hipError_t e) { return e == hipSuccess ? R3_OK : R3_ERR_HIP; }

// Scratch of r3_permute_static: a fixed array in every device's copy of this code object, held until
// the process ends.  `scratch` is a host-side stand-in for the symbol, not a device address; the
// device address is looked up once per device (static_scratch) and only that pointer is ever handed
// to a kernel.
constexpr int kMaxDevices = 64;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[R3_STATIC_SCRATCH_BYTES];
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mu;

int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return R3_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lk(g_scratch_mu);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return R3_ERR_HIP;
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return R3_OK;
}

}  // namespace

extern "C" {

const char *r3_version(void) { return "r3-mi355x 0.1 (gfx950, bf16 MFMA + f32 SIMT)"; }

size_t r3_workspace_bytes(const r3_layer_desc *desc, r3_op op) {
    Dims m;
    if (check_desc(desc, m) != R3_OK) return 0;
    switch (op) {
        case R3_OP_REPLAY_GATE: return align_up((size_t)m.T * m.E * sizeof(float), 256);
        case R3_OP_PERMUTE: return permute_ws_bytes(m.T, m.E, m.K);
        case R3_OP_GROUPED_FFN: return use_mfma_ffn(m) ? mfma_tiles_bytes(m.S, m.E) : 0;
        case R3_OP_BACKWARD: return bwd_layout(m).total;
        case R3_OP_FORWARD: return fwd_layout(m).total;
    }
    return 0;
}

int r3_record_topk(const r3_layer_desc *desc, const float *logits, int64_t ld, void *idx_out,
                   int32_t *status_word, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (!logits || !idx_out || ld < m.E || !aligned(logits, 4)) return R3_ERR_INVALID_ARG;
    if (m.idx == R3_IDX_U16 && !aligned(idx_out, 2)) return R3_ERR_INVALID_ARG;
    return hip_rc(launch_record_topk(m.T, m.E, m.K, logits, ld, idx_out, m.idx, m.stride, status_word,
                                     (hipStream_t)stream));
}

int r3_replay_gate(const r3_layer_desc *desc, const void *x, const void *W_r, const float *bias,
                   const void *idx, float *gates, float *logits_out, int64_t *agree_out,
                   int32_t *status_word, void *ws, size_t ws_bytes, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (!x || !W_r || !idx || !gates) return R3_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(W_r, 16) || !aligned(gates, 4) || (logits_out && !aligned(logits_out, 16)) ||
        (bias && !aligned(bias, 16)) || (agree_out && !aligned(agree_out, 8)) ||
        (status_word && !aligned(status_word, 4)) || (m.idx == R3_IDX_U16 && !aligned(idx, 2)))
        return R3_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    // one launch: the logits stay in the work-group that made them (no workspace needed)
    if (use_mfma_router(m) && mfma_gate_fused_supported(m.d, m.E, m.K, agree_out != nullptr))
        return hip_rc(mfma_gate_fused(m.T, m.d, m.E, m.K, x, W_r, bias, idx, m.idx, m.stride, gates, logits_out,
                                      agree_out, status_word, s));
    float *logits = logits_out;
    if (!logits) {
        if (!ws || ws_bytes < r3_workspace_bytes(desc, R3_OP_REPLAY_GATE) || !aligned(ws, 256))
            return R3_ERR_WORKSPACE;
        logits = (float *)ws;
    }
    hipError_t e;
    if (use_mfma_router(m)) e = mfma_router_logits(m.T, m.d, m.E, x, W_r, bias, logits, s);
    else e = simt_router_logits(m.T, m.d, m.E, m.act, x, W_r, bias, logits, s);
    if (e != hipSuccess) return R3_ERR_HIP;
    e = launch_gate(m.T, m.E, m.K, logits, idx, m.idx, m.stride, gates, status_word, s);
    if (e != hipSuccess) return R3_ERR_HIP;
    if (agree_out) e = launch_agreement(m.T, m.E, m.K, logits, idx, m.idx, m.stride, agree_out, s);
    return hip_rc(e);
}

int r3_permute(const r3_layer_desc *desc, const void *x, const void *idx, int32_t *counts,
               int32_t *offsets, int32_t *inv_perm, int32_t *perm, void *Xp, int32_t *status_word,
               void *ws, size_t ws_bytes, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (!idx || !counts || !offsets || !inv_perm || !perm || (Xp && !x)) return R3_ERR_INVALID_ARG;
    if ((Xp && (!aligned(Xp, 16) || !aligned(x, 16))) || !aligned(counts, 4) || !aligned(offsets, 4) ||
        !aligned(inv_perm, 4) || !aligned(perm, 4))
        return R3_ERR_INVALID_ARG;
    if (!ws || ws_bytes < permute_ws_bytes(m.T, m.E, m.K) || !aligned(ws, 256)) return R3_ERR_WORKSPACE;
    return hip_rc(launch_permute(m.T, m.d, m.E, m.K, m.eb, x, idx, m.idx, m.stride, counts, offsets, inv_perm,
                                 perm, Xp, status_word, ws, (hipStream_t)stream));
}

int r3_permute_static(const r3_layer_desc *desc, const void *x, const void *idx, int32_t *counts,
                      int32_t *offsets, int32_t *inv_perm, int32_t *perm, void *Xp, int32_t *status_word,
                      void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (permute_ws_bytes(m.T, m.E, m.K) > (size_t)R3_STATIC_SCRATCH_BYTES) return R3_ERR_UNSUPPORTED;
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    return r3_permute(desc, x, idx, counts, offsets, inv_perm, perm, Xp, status_word, ws,
                      (size_t)R3_STATIC_SCRATCH_BYTES, stream);
}

int r3_grouped_ffn(const r3_layer_desc *desc, const void *Xp, const void *x, const int32_t *perm,
                   const int32_t *offsets, const void *W_gate, const void *W_up, const void *W_down, void *Yp,
                   void *H, void *FA_save, void *FB_save, void *ws, size_t ws_bytes, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (!offsets || !W_gate || !W_up || !W_down || !Yp || !H || ((FA_save == nullptr) != (FB_save == nullptr)))
        return R3_ERR_INVALID_ARG;
    if (!Xp && (!x || !perm)) return R3_ERR_INVALID_ARG;   // rows come from Xp, or from x through perm
    if (!aligned(Xp, 16) || !aligned(x, 16) || !aligned(perm, 4) || !aligned(W_gate, 16) || !aligned(W_up, 16) ||
        !aligned(W_down, 16) || !aligned(Yp, 16) || !aligned(H, 16) || !aligned(FA_save, 16) || !aligned(FB_save, 16))
        return R3_ERR_INVALID_ARG;
    const void *rows = Xp ? Xp : x;
    const int32_t *via = Xp ? nullptr : perm;
    if (via && (int64_t)m.T * m.d * m.eb > 0x7fffffffLL) return R3_ERR_UNSUPPORTED;   // 32-bit row offsets
    hipStream_t s = (hipStream_t)stream;
    if (use_mfma_ffn(m)) {
        if (!ws || ws_bytes < mfma_tiles_bytes(m.S, m.E) || !aligned(ws, 256)) return R3_ERR_WORKSPACE;
        int32_t *tiles = (int32_t *)ws;
        if (mfma_build_tiles(m.E, offsets, tiles, -1, s) != hipSuccess) return R3_ERR_HIP;
        return hip_rc(mfma_ffn_forward(m.S, m.d, m.E, m.F, rows, via, m.K, m.T, offsets, tiles, W_gate, W_up, W_down,
                                       Yp, H, FA_save, FB_save, nullptr, s));
    }
    if (simt_ffn1((int)m.S, m.d, m.E, m.F, m.act, rows, via, m.K, offsets, W_gate, W_up, H, FA_save, FB_save, nullptr,
                  s) !=
        hipSuccess)
        return R3_ERR_HIP;
    return hip_rc(simt_ffn2((int)m.S, m.d, m.E, m.F, m.act, H, offsets, W_down, Yp, s));
}

int r3_combine(const r3_layer_desc *desc, const void *Yp, const float *gates, const int32_t *inv_perm,
               void *y, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (!Yp || !gates || !inv_perm || !y) return R3_ERR_INVALID_ARG;
    if (!aligned(Yp, 16) || !aligned(y, 16) || !aligned(gates, 4) || !aligned(inv_perm, 4))
        return R3_ERR_INVALID_ARG;
    return hip_rc(launch_combine(m.T, m.d, m.K, m.act, Yp, gates, inv_perm, y, (hipStream_t)stream));
}

int r3_moe_forward(const r3_layer_desc *desc, const void *x, const void *W_r, const float *bias, const void *idx,
                   const void *W_gate, const void *W_up, const void *W_down, void *y, float *gates, int32_t *counts,
                   int32_t *offsets, int32_t *inv_perm, int32_t *perm, void *Yp, void *H, void *FA_save,
                   void *FB_save, float *logits_out, int64_t *agree_out, int32_t *status_word, void *ws,
                   size_t ws_bytes, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (!x || !W_gate || !W_up || !W_down || !y || !Yp || !H || ((FA_save == nullptr) != (FB_save == nullptr)))
        return R3_ERR_INVALID_ARG;   // (the other pointers are checked by the steps)
    if (!aligned(y, 16) || !aligned(Yp, 16) || !aligned(H, 16) || !aligned(FA_save, 16) || !aligned(FB_save, 16) ||
        !aligned(W_gate, 16) || !aligned(W_up, 16) || !aligned(W_down, 16))
        return R3_ERR_INVALID_ARG;
    if ((int64_t)m.T * m.d * m.eb > 0x7fffffffLL) return R3_ERR_UNSUPPORTED;   // rows are read through perm
    const FwdWs w = fwd_layout(m);
    if (!ws || ws_bytes < w.total || !aligned(ws, 256)) return R3_ERR_WORKSPACE;
    char *base = (char *)ws;
    hipStream_t s = (hipStream_t)stream;
    r3_layer_desc plain = *desc;
    plain.flags = 0;
    rc = r3_replay_gate(&plain, x, W_r, bias, idx, gates, logits_out, agree_out, status_word, base + w.gate,
                        w.perm - w.gate, stream);
    if (rc) return rc;
    rc = r3_permute(&plain, nullptr, idx, counts, offsets, inv_perm, perm, nullptr, status_word, base + w.perm,
                    w.ffn - w.perm, stream);
    if (rc) return rc;
    // the gate of every expert-sorted row: the first contraction's epilogue scales H with it, so the
    // down projection yields gated rows and the combination is a plain sum of each token's K rows
    int32_t *tok = (int32_t *)(base + w.tok);
    float *grow = (float *)(base + w.grow);
    if (use_mfma_ffn(m)) {
        int32_t *tiles = (int32_t *)(base + w.ffn);
        if (mfma_build_tiles_and_row_tokens(m.E, offsets, tiles, -1, (int)m.S, m.K, perm, gates, tok, grow, s) !=
            hipSuccess)
            return R3_ERR_HIP;
        if (mfma_ffn_forward(m.S, m.d, m.E, m.F, x, perm, m.K, m.T, offsets, tiles, W_gate, W_up, W_down, Yp, H,
                             FA_save, FB_save, grow, s) != hipSuccess)
            return R3_ERR_HIP;
    } else {
        if (mfma_row_tokens((int)m.S, m.K, perm, gates, tok, grow, s) != hipSuccess) return R3_ERR_HIP;
        if (simt_ffn1((int)m.S, m.d, m.E, m.F, m.act, x, perm, m.K, offsets, W_gate, W_up, H, FA_save, FB_save, grow,
                      s) != hipSuccess)
            return R3_ERR_HIP;
        if (simt_ffn2((int)m.S, m.d, m.E, m.F, m.act, H, offsets, W_down, Yp, s) != hipSuccess) return R3_ERR_HIP;
    }
    return hip_rc(launch_combine(m.T, m.d, m.K, m.act, Yp, nullptr, inv_perm, y, s));
}

int r3_moe_backward(const r3_layer_desc *desc, const void *dy, const void *x, const void *W_r,
                    const void *idx, const float *gates, const int32_t *inv_perm, const int32_t *perm,
                    const int32_t *offsets, const void *Xp, const void *FA, const void *FB, const void *H,
                    const void *Yp, const void *W_gate, const void *W_up, const void *W_down, void *dx,
                    float *dW_r, float *dW_gate, float *dW_up, float *dW_down, float *dbias,
                    int accumulate, void *ws, size_t ws_bytes, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    const bool mf = use_mfma_ffn(m);
    const bool gated = (m.flags & R3_FLAG_GATED_H) != 0;   // H = g H and Yp = g o, as r3_moe_forward leaves them
    const void *ptrs[] = {dy, x, W_r, idx, gates, inv_perm, offsets, FA, FB, H, W_gate, W_up, W_down,
                          dx, dW_r, dW_gate, dW_up, dW_down};
    for (const void *p : ptrs)
        if (!p) return R3_ERR_INVALID_ARG;
    const void *a16[] = {dy, x, W_r, Xp, FA, FB, H, Yp, W_gate, W_up, W_down, dx, dW_r, dW_gate, dW_up, dW_down};
    for (const void *p : a16)
        if (!aligned(p, 16)) return R3_ERR_INVALID_ARG;
    if (accumulate != 0 && accumulate != 1) return R3_ERR_INVALID_ARG;
    if (mf) {
        // rows of dy (and of x when there is no Xp) are read through perm inside the tile loads
        if (!perm || !aligned(perm, 4)) return R3_ERR_INVALID_ARG;
        if ((int64_t)m.T * m.d * m.eb >= (1ll << 31)) return R3_ERR_UNSUPPORTED;   // 32-bit row offsets
    } else if (!Yp || ((!Xp || gated) && (!perm || !aligned(perm, 4)))) {
        return R3_ERR_INVALID_ARG;   // the plain kernels need Yp, and Xp or perm (perm after r3_moe_forward)
    }
    const BwdWs w = bwd_layout(m);
    if (!ws || ws_bytes < w.total || !aligned(ws, 256)) return R3_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *base = (char *)ws;
    void *dXp = base + w.dXp, *ds = base + w.ds, *WrT = base + w.WrT, *dA = base + w.dA, *dB = base + w.dB;
    float *dz = (float *)(base + w.dz);
    const int S = (int)m.S;
    hipError_t e;

    if (mf) {
        // experts first: the gradient GEMM of the down projection reads dy through the row -> token
        // list and leaves the dot products the masked softmax needs (no g*dy copy, no read of Yp)
        int32_t *tiles = (int32_t *)(base + w.tiles), *tok = (int32_t *)(base + w.tok);
        float *grow = (float *)(base + w.grow), *wpart = (float *)(base + w.wpart);
        void *Hg = gated ? nullptr : base + w.Hg;
        // a heavily loaded expert's weight-gradient reductions are cut into parts; their partial products
        // sit in the dXp buffer, which nothing uses before the parts are summed (dW_down's first, then, in
        // the same place, dW_gate's and dW_up's side by side)
        const size_t slot_bytes = 2 * (size_t)m.F * m.d * sizeof(float);
        const int split = mfma_wgrad_split_rows(m.S, (m.F / 256) * (m.d / 256), (size_t)m.S * m.d * m.eb, slot_bytes);
        if (mfma_build_tiles_and_row_tokens(m.E, offsets, tiles, split, S, m.K, perm, gates, tok, grow, s) != hipSuccess)
            return R3_ERR_HIP;
        if (mfma_ffn_dh(m.S, m.d, m.E, m.F, dy, tok, m.T, grow, offsets, tiles, W_down, FA, FB, H, dA, dB, Hg, wpart,
                        s) != hipSuccess)
            return R3_ERR_HIP;
        if (launch_gate_backward_parts(m.T, m.E, m.K, row_parts(m), wpart, gates, inv_perm, idx, m.idx, m.stride, dz,
                                       ds, s) != hipSuccess)
            return R3_ERR_HIP;
        if (mfma_wgrad(m.E, m.F, m.d, gated ? H : Hg, dy, tok, m.T, tiles, 2, dW_down, split ? (float *)dXp : nullptr,
                       accumulate, s) != hipSuccess)
            return R3_ERR_HIP;
        if (mfma_wgrad_pair(m.E, m.d, m.F, Xp ? Xp : x, Xp ? nullptr : tok, m.T, dA, dB, tiles, 3, dW_gate, dW_up,
                            split ? (float *)dXp : nullptr, accumulate, s) != hipSuccess)
            return R3_ERR_HIP;
        if (mfma_ffn_dxp(m.S, m.d, m.E, m.F, dA, dB, offsets, tiles, W_gate, W_up, dXp, s) != hipSuccess)
            return R3_ERR_HIP;
    } else {
        // combine and masked softmax:  dYp = g*dy per slot, dz, dense ds
        void *dYp = dXp;  // dYp is dead once dW_down and dH are done
        if (launch_gate_backward(m.T, m.d, m.E, m.K, m.act, dy, Yp, gates, inv_perm, idx, m.idx, m.stride, dYp, dz,
                                 ds, gated ? 1 : 0, s) != hipSuccess)
            return R3_ERR_HIP;
        if (simt_dh(S, m.d, m.E, m.F, m.act, dYp, offsets, W_down, FA, FB, dA, dB, s) != hipSuccess) return R3_ERR_HIP;
        const int32_t *tok = nullptr;
        if (gated || !Xp) {   // rows of dy / x through the row -> token list
            int32_t *t = (int32_t *)(base + w.tok);
            if (mfma_row_tokens(S, m.K, perm, nullptr, t, nullptr, s) != hipSuccess) return R3_ERR_HIP;
            tok = t;
        }
        // gated: H is g H already, so its partner is the plain dy row, not g dy
        e = gated ? simt_wgrad(m.E, m.F, m.d, m.act, H, nullptr, dy, tok, offsets, dW_down, accumulate, s)
                  : simt_wgrad(m.E, m.F, m.d, m.act, H, nullptr, dYp, nullptr, offsets, dW_down, accumulate, s);
        if (e != hipSuccess) return R3_ERR_HIP;
        const void *rows = Xp ? Xp : x;          // the token rows, gathered or through the list
        const int32_t *rtok = Xp ? nullptr : tok;
        if (simt_wgrad(m.E, m.d, m.F, m.act, rows, rtok, dA, nullptr, offsets, dW_gate, accumulate, s) != hipSuccess)
            return R3_ERR_HIP;
        if (simt_wgrad(m.E, m.d, m.F, m.act, rows, rtok, dB, nullptr, offsets, dW_up, accumulate, s) != hipSuccess)
            return R3_ERR_HIP;
        if (simt_dxp(S, m.d, m.E, m.F, m.act, dA, dB, offsets, W_gate, W_up, dXp, s) != hipSuccess) return R3_ERR_HIP;
    }
    // router:  dW_r = x^T ds, dbias = column sums
    if (use_mfma_router(m)) e = mfma_dwr(m.T, m.d, m.E, x, ds, (float *)(base + w.part), dW_r, accumulate, s);
    else e = simt_dwr(m.T, m.d, m.E, m.act, x, ds, dW_r, accumulate, s);
    if (e != hipSuccess) return R3_ERR_HIP;
    if (dbias && launch_colsum(m.T, m.E, m.act, ds, dbias, accumulate, s) != hipSuccess) return R3_ERR_HIP;
    if (launch_transpose(m.d, m.E, m.act, W_r, WrT, s) != hipSuccess) return R3_ERR_HIP;
    // dx = un-permuted expert gradients + router term
    return hip_rc(launch_dx_finish(m.T, m.d, m.E, m.K, m.act, dXp, WrT, dz, inv_perm, idx, m.idx, m.stride, dx,
                                   s));
}

int r3_routing_diff(const r3_layer_desc *desc, int L, const void *idx_a, const void *idx_b, int64_t layer_stride,
                    const int32_t *seq_offsets, int nseq, int64_t *router_hist, int32_t *token_choices,
                    int32_t *token_routers, double *seq_mean, void *stream) {
    Dims m;
    int rc = check_desc(desc, m);
    if (rc) return rc;
    if (L <= 0 || !idx_a || !idx_b || layer_stride < m.K || !router_hist || !token_choices || !token_routers ||
        nseq < 0 || (seq_mean && (!seq_offsets || nseq == 0)))
        return R3_ERR_INVALID_ARG;
    if (!aligned(router_hist, 8) || !aligned(token_choices, 4) || !aligned(token_routers, 4) ||
        (seq_mean && (!aligned(seq_mean, 8) || !aligned(seq_offsets, 4))) ||
        (m.idx == R3_IDX_U16 && (!aligned(idx_a, 2) || !aligned(idx_b, 2))))
        return R3_ERR_INVALID_ARG;
    return hip_rc(launch_routing_diff(m.T, m.K, L, idx_a, idx_b, m.idx, m.stride, layer_stride, seq_offsets,
                                      seq_mean ? nseq : 0, router_hist, token_choices, token_routers, seq_mean,
                                      (hipStream_t)stream));
}

size_t r3_policy_workspace_bytes(void) { return policy_ws_bytes(); }

int r3_policy_discrepancy(int64_t n, const float *logp_train, const float *logp_infer, int ntau, const float *tau,
                          double *kl_out, double *frac_out, void *ws, size_t ws_bytes, void *stream) {
    if (n < 0 || ntau < 0 || ntau > policy_max_tau() || !kl_out || (ntau > 0 && (!tau || !frac_out)) ||
        (n > 0 && (!logp_train || !logp_infer)))
        return R3_ERR_INVALID_ARG;
    for (int i = 0; i < ntau; ++i)
        if (!(tau[i] >= 1.0f)) return R3_ERR_INVALID_ARG;
    if (!aligned(logp_train, 4) || !aligned(logp_infer, 4) || !aligned(kl_out, 8) || (frac_out && !aligned(frac_out, 8)))
        return R3_ERR_INVALID_ARG;
    if (!ws || ws_bytes < policy_ws_bytes() || !aligned(ws, 256)) return R3_ERR_WORKSPACE;
    return hip_rc(launch_policy_discrepancy(n, logp_train, logp_infer, ntau, tau, kl_out, frac_out, ws,
                                            (hipStream_t)stream));
}

static int check_cache(int idx_dtype, int L, int K, int P, const void *pages, int64_t num_pages,
                       const int32_t *block_table, int nseq, int max_blocks, int &idx_bytes) {
    if (idx_dtype != R3_IDX_U8 && idx_dtype != R3_IDX_U16) return R3_ERR_INVALID_ARG;
    idx_bytes = idx_dtype == R3_IDX_U8 ? 1 : 2;
    if (L <= 0 || K <= 0 || P <= 0 || !pages || num_pages <= 0 || !block_table || nseq <= 0 || max_blocks <= 0)
        return R3_ERR_INVALID_ARG;
    if (!aligned(pages, idx_bytes) || !aligned(block_table, 4)) return R3_ERR_INVALID_ARG;
    // rows of the pool are addressed as page*P + slot in 64 bits; positions as int32
    if ((int64_t)max_blocks * P > 0x7fffffffll || (int64_t)L * K > (1 << 20)) return R3_ERR_UNSUPPORTED;
    return R3_OK;
}

int r3_mask_cache_append(int idx_dtype, int L, int K, int P, void *pages, int64_t num_pages,
                         const int32_t *block_table, int nseq, int max_blocks, int64_t n, const int32_t *seq_id,
                         const int32_t *position, const void *idx_new, int64_t layer_stride, int64_t token_stride,
                         int32_t *status_word, void *stream) {
    int ib = 0;
    int rc = check_cache(idx_dtype, L, K, P, pages, num_pages, block_table, nseq, max_blocks, ib);
    if (rc) return rc;
    if (n < 0 || (n > 0 && (!seq_id || !position || !idx_new)) || layer_stride < 0 || token_stride < 0)
        return R3_ERR_INVALID_ARG;
    if (n > 0x7fffffffll) return R3_ERR_UNSUPPORTED;
    if (!aligned(seq_id, 4) || !aligned(position, 4) || !aligned(idx_new, ib) || (status_word && !aligned(status_word, 4)))
        return R3_ERR_INVALID_ARG;
    return hip_rc(launch_cache_append(ib, L, K, P, pages, num_pages, block_table, nseq, max_blocks, n, seq_id,
                                      position, idx_new, layer_stride, token_stride, status_word,
                                      (hipStream_t)stream));
}

int r3_mask_cache_gather(int idx_dtype, int L, int K, int P, const void *pages, int64_t num_pages,
                         const int32_t *block_table, int nseq, int max_blocks, const int32_t *seq_start, int64_t T,
                         void *out, int32_t *status_word, void *stream) {
    int ib = 0;
    int rc = check_cache(idx_dtype, L, K, P, pages, num_pages, block_table, nseq, max_blocks, ib);
    if (rc) return rc;
    if (T < 0 || T > 0x7fffffffll - 64 || !seq_start || (T > 0 && !out)) return R3_ERR_INVALID_ARG;
    if (!aligned(seq_start, 4) || !aligned(out, ib) || (status_word && !aligned(status_word, 4)))
        return R3_ERR_INVALID_ARG;
    return hip_rc(launch_cache_gather(ib, L, K, P, pages, num_pages, block_table, nseq, max_blocks, seq_start,
                                      (int)T, out, status_word, (hipStream_t)stream));
}

}  // extern "C"
