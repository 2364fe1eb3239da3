"""Thin ctypes binding over libr3.so (the C ABI in include/r3.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the layer runs in the library's kernels.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libr3.so")

BF16, F32 = 0, 1
IDX_U8, IDX_U16 = 0, 1
OP_REPLAY_GATE, OP_PERMUTE, OP_GROUPED_FFN, OP_BACKWARD, OP_FORWARD = 0, 1, 2, 3, 4
FLAG_GATED_H = 1
DATA_IDX_RANGE, DATA_IDX_DUP, DATA_NONFINITE = 1, 2, 4
_STATUS = {1: "R3_ERR_INVALID_ARG", 2: "R3_ERR_UNSUPPORTED", 3: "R3_ERR_WORKSPACE", 4: "R3_ERR_HIP"}

EXPORTS = ["r3_version", "r3_workspace_bytes", "r3_record_topk", "r3_replay_gate", "r3_permute",
           "r3_permute_static", "r3_grouped_ffn", "r3_combine", "r3_moe_forward", "r3_moe_backward", "r3_profile_enable", "r3_profile_tags",
           "r3_profile_name", "r3_profile_read", "r3_profile_copy",
           "r3_profile_mfma", "r3_profile_mfma_flops", "r3_profile_gemm_mix", "r3_routing_diff", "r3_policy_discrepancy",
           "r3_policy_workspace_bytes", "r3_mask_cache_append", "r3_mask_cache_gather"]


class LayerDesc(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("E", C.c_int32), ("K", C.c_int32),
                ("F", C.c_int32), ("act", C.c_int32), ("idx", C.c_int32), ("flags", C.c_int32),
                ("idx_token_stride", C.c_int64)]


class R3Error(RuntimeError):
    pass


_lib = None


def lib():
    """Load libr3.so; build it first with paper_2510_11370_amd/build.py."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise R3Error("libr3.so is not built: run `python -m paper_2510_11370_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        L.r3_version.restype = C.c_char_p
        L.r3_workspace_bytes.restype = C.c_size_t
        L.r3_workspace_bytes.argtypes = [C.POINTER(LayerDesc), C.c_int]
        for name in EXPORTS[2:]:
            getattr(L, name).restype = C.c_int
        L.r3_profile_name.restype = C.c_char_p
        L.r3_profile_mfma_flops.restype = C.c_double
        L.r3_policy_workspace_bytes.restype = C.c_size_t
        _lib = L
    return _lib


def desc(T, d, E, K, F, act="bf16", idx_dtype=None, idx_token_stride=0):
    if idx_dtype is None:
        idx_dtype = torch.uint8 if E <= 256 else torch.uint16
    return LayerDesc(T, d, E, K, F, BF16 if act in ("bf16", torch.bfloat16) else F32,
                     IDX_U8 if idx_dtype == torch.uint8 else IDX_U16, 0, idx_token_stride)


def act_dtype(D):
    return torch.bfloat16 if D.act == BF16 else torch.float32


def idx_torch_dtype(D):
    return torch.uint8 if D.idx == IDX_U8 else torch.uint16


def _p(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc != 0:
        raise R3Error("%s failed: %s" % (what, _STATUS.get(rc, rc)))


def workspace_bytes(D, op):
    return int(lib().r3_workspace_bytes(C.byref(D), op))


def workspace(D, op, device="cuda"):
    """A fresh workspace tensor for `op` (torch's allocator aligns to 256 bytes)."""
    return torch.empty(max(workspace_bytes(D, op), 256), dtype=torch.uint8, device=device)


def record_topk(D, logits, idx_out, status=None):
    _check(lib().r3_record_topk(C.byref(D), _p(logits), C.c_int64(logits.stride(0)), _p(idx_out),
                                _p(status), _stream()), "r3_record_topk")


def replay_gate(D, x, W_r, idx, gates, bias=None, logits_out=None, agree_out=None, status=None, ws=None):
    _check(lib().r3_replay_gate(C.byref(D), _p(x), _p(W_r), _p(bias), _p(idx), _p(gates), _p(logits_out),
                                _p(agree_out), _p(status), _p(ws),
                                C.c_size_t(0 if ws is None else ws.numel()), _stream()), "r3_replay_gate")


def permute(D, x, idx, counts, offsets, inv_perm, perm, Xp, ws, status=None):
    _check(lib().r3_permute(C.byref(D), _p(x), _p(idx), _p(counts), _p(offsets), _p(inv_perm), _p(perm),
                            _p(Xp), _p(status), _p(ws), C.c_size_t(ws.numel()), _stream()), "r3_permute")


def permute_static(D, x, idx, counts, offsets, inv_perm, perm, Xp, status=None):
    """r3_permute with the library's own fixed scratch array (allocates nothing, takes no workspace)."""
    _check(lib().r3_permute_static(C.byref(D), _p(x), _p(idx), _p(counts), _p(offsets), _p(inv_perm), _p(perm),
                                   _p(Xp), _p(status), _stream()), "r3_permute_static")


def grouped_ffn(D, Xp, offsets, W_gate, W_up, W_down, Yp, H, A_save=None, B_save=None, ws=None, x=None, perm=None):
    """Xp=None with x and perm: the token rows are gathered inside the first contraction.
    A_save, B_save receive the backward's two factors FA = B silu'(A) and FB = silu(A) (see include/r3.h)."""
    _check(lib().r3_grouped_ffn(C.byref(D), _p(Xp), _p(x), _p(perm), _p(offsets), _p(W_gate), _p(W_up), _p(W_down), _p(Yp),
                                _p(H), _p(A_save), _p(B_save), _p(ws),
                                C.c_size_t(0 if ws is None else ws.numel()), _stream()), "r3_grouped_ffn")


def combine(D, Yp, gates, inv_perm, y):
    _check(lib().r3_combine(C.byref(D), _p(Yp), _p(gates), _p(inv_perm), _p(y), _stream()), "r3_combine")


def moe_forward(D, x, W_r, idx, W_gate, W_up, W_down, y, gates, counts, offsets, inv_perm, perm, Yp, H, ws,
                FA_save=None, FB_save=None, bias=None, logits_out=None, agree_out=None, status=None):
    """The replayed forward in one call; H and Yp come out gate-scaled (differentiate with gated_desc(D))."""
    _check(lib().r3_moe_forward(C.byref(D), _p(x), _p(W_r), _p(bias), _p(idx), _p(W_gate), _p(W_up), _p(W_down),
                                _p(y), _p(gates), _p(counts), _p(offsets), _p(inv_perm), _p(perm), _p(Yp), _p(H),
                                _p(FA_save), _p(FB_save), _p(logits_out), _p(agree_out), _p(status), _p(ws),
                                C.c_size_t(ws.numel()), _stream()), "r3_moe_forward")


def gated_desc(D):
    """A copy of D with R3_FLAG_GATED_H set: what r3_moe_backward takes after r3_moe_forward."""
    return LayerDesc(D.T, D.d, D.E, D.K, D.F, D.act, D.idx, FLAG_GATED_H, D.idx_token_stride)


def moe_backward(D, dy, x, W_r, idx, gates, inv_perm, perm, offsets, Xp, A, B, H, Yp, W_gate, W_up, W_down,
                 dx, dW_r, dW_gate, dW_up, dW_down, ws, dbias=None, accumulate=False):
    _check(lib().r3_moe_backward(C.byref(D), _p(dy), _p(x), _p(W_r), _p(idx), _p(gates), _p(inv_perm),
                                 _p(perm), _p(offsets), _p(Xp), _p(A), _p(B), _p(H), _p(Yp), _p(W_gate),
                                 _p(W_up), _p(W_down), _p(dx), _p(dW_r), _p(dW_gate), _p(dW_up), _p(dW_down),
                                 _p(dbias), C.c_int(1 if accumulate else 0), _p(ws), C.c_size_t(ws.numel()),
                                 _stream()), "r3_moe_backward")


def routing_diff(D, L, idx_a, idx_b, layer_stride, router_hist, token_choices, token_routers, seq_offsets=None,
                 seq_mean=None):
    nseq = 0 if seq_offsets is None else seq_offsets.numel() - 1
    _check(lib().r3_routing_diff(C.byref(D), C.c_int(L), _p(idx_a), _p(idx_b), C.c_int64(layer_stride),
                                 _p(seq_offsets), C.c_int(nseq), _p(router_hist), _p(token_choices),
                                 _p(token_routers), _p(seq_mean), _stream()), "r3_routing_diff")


def policy_discrepancy(logp_train, logp_infer, taus, kl_out, frac_out, ws=None):
    """taus: host floats (>= 1); kl_out [1], frac_out [len(taus)]: device float64."""
    if ws is None:
        ws = torch.empty(lib().r3_policy_workspace_bytes(), dtype=torch.uint8, device=logp_train.device)
    tau = (C.c_float * max(len(taus), 1))(*taus)
    _check(lib().r3_policy_discrepancy(C.c_int64(logp_train.numel()), _p(logp_train), _p(logp_infer),
                                       C.c_int(len(taus)), tau, _p(kl_out), _p(frac_out), _p(ws),
                                       C.c_size_t(ws.numel()), _stream()), "r3_policy_discrepancy")


def _idx_code(t):
    return IDX_U8 if t.dtype == torch.uint8 else IDX_U16


def mask_cache_append(pages, block_table, seq_id, position, idx_new, layer_stride, token_stride, status=None):
    """pages [num_pages,P,L,K]; block_table int32 [nseq,max_blocks]; idx_new: element (l,i,k) at
    l*layer_stride + i*token_stride + k."""
    num_pages, P, L, K = pages.shape
    _check(lib().r3_mask_cache_append(C.c_int(_idx_code(pages)), C.c_int(L), C.c_int(K), C.c_int(P), _p(pages),
                                      C.c_int64(num_pages), _p(block_table), C.c_int(block_table.shape[0]),
                                      C.c_int(block_table.shape[1]), C.c_int64(seq_id.numel()), _p(seq_id),
                                      _p(position), _p(idx_new), C.c_int64(layer_stride), C.c_int64(token_stride),
                                      _p(status), _stream()), "r3_mask_cache_append")


def mask_cache_gather(pages, block_table, seq_start, out, status=None):
    """out [L,T,K]: the layer-major record of the packed batch described by seq_start (int32 [nseq+1])."""
    num_pages, P, L, K = pages.shape
    _check(lib().r3_mask_cache_gather(C.c_int(_idx_code(pages)), C.c_int(L), C.c_int(K), C.c_int(P), _p(pages),
                                      C.c_int64(num_pages), _p(block_table), C.c_int(block_table.shape[0]),
                                      C.c_int(block_table.shape[1]), _p(seq_start), C.c_int64(out.shape[1]),
                                      _p(out), _p(status), _stream()), "r3_mask_cache_gather")


class LayerBuffers:
    """Caller-owned buffers of one layer (everything the C ABI reads or writes)."""

    def __init__(self, D, device="cuda", backward=True, gathered_copy=True):
        """gathered_copy=False: no Xp; the expert GEMMs read token rows from x through perm (bf16 MFMA shapes)."""
        T, d, E, K, F = D.T, D.d, D.E, D.K, D.F
        S = T * K
        a = act_dtype(D)
        e = lambda *s, dt=a: torch.empty(*s, dtype=dt, device=device)
        self.D = D
        self.gates = e(T, K, dt=torch.float32)
        self.counts = e(E, dt=torch.int32)
        self.offsets = e(E + 1, dt=torch.int32)
        self.inv_perm = e(S, dt=torch.int32)
        self.perm = e(S, dt=torch.int32)
        self.Xp = e(S, d) if gathered_copy else None
        self.Yp, self.H, self.y = e(S, d), e(S, F), e(T, d)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.ws_gate = workspace(D, OP_REPLAY_GATE, device)
        self.ws_perm = workspace(D, OP_PERMUTE, device)
        self.ws_ffn = workspace(D, OP_GROUPED_FFN, device)
        self.ws_fwd = None         # made on first use by forward_one_call()
        self.gated = False         # whether H / Yp hold gate-scaled rows (set by the forward that filled them)
        self.A = self.B = None             # the saved factors FA = B silu'(A), FB = silu(A)
        if backward:
            self.A, self.B = e(S, F), e(S, F)
            self.dx = e(T, d)
            self.dW_r = e(d, E, dt=torch.float32)
            self.dW_gate = e(E, d, F, dt=torch.float32)
            self.dW_up = e(E, d, F, dt=torch.float32)
            self.dW_down = e(E, F, d, dt=torch.float32)
            self.ws_bwd = workspace(D, OP_BACKWARD, device)


def forward(buf, x, W_r, idx, W_gate, W_up, W_down, bias=None, logits_out=None, agree_out=None):
    """The replayed forward as four C calls: gate -> permute -> grouped FFN -> combine."""
    D = buf.D
    replay_gate(D, x, W_r, idx, buf.gates, bias=bias, logits_out=logits_out, agree_out=agree_out,
                status=buf.status, ws=buf.ws_gate)
    permute(D, x, idx, buf.counts, buf.offsets, buf.inv_perm, buf.perm, buf.Xp, buf.ws_perm, status=buf.status)
    grouped_ffn(D, buf.Xp, buf.offsets, W_gate, W_up, W_down, buf.Yp, buf.H, buf.A, buf.B, ws=buf.ws_ffn,
                x=x, perm=buf.perm)
    combine(D, buf.Yp, buf.gates, buf.inv_perm, buf.y)
    buf.gated = False
    return buf.y


def forward_one_call(buf, x, W_r, idx, W_gate, W_up, W_down, bias=None, logits_out=None, agree_out=None):
    """The replayed forward as one C call (r3_moe_forward): buf.H and buf.Yp then hold gate-scaled rows."""
    D = buf.D
    if buf.ws_fwd is None:
        buf.ws_fwd = workspace(D, OP_FORWARD, buf.status.device)
    moe_forward(D, x, W_r, idx, W_gate, W_up, W_down, buf.y, buf.gates, buf.counts, buf.offsets, buf.inv_perm,
                buf.perm, buf.Yp, buf.H, buf.ws_fwd, FA_save=buf.A, FB_save=buf.B, bias=bias, logits_out=logits_out,
                agree_out=agree_out, status=buf.status)
    buf.gated = True
    return buf.y


def backward(buf, dy, x, W_r, idx, W_gate, W_up, W_down, dbias=None, accumulate=False):
    """r3_moe_backward on the buffers' saved tensors (told whether the last forward left them gate-scaled)."""
    D = gated_desc(buf.D) if buf.gated else buf.D
    moe_backward(D, dy, x, W_r, idx, buf.gates, buf.inv_perm, buf.perm, buf.offsets,
                 None if buf.gated else buf.Xp, buf.A, buf.B,
                 buf.H, buf.Yp, W_gate, W_up, W_down, buf.dx, buf.dW_r, buf.dW_gate, buf.dW_up, buf.dW_down,
                 buf.ws_bwd, dbias=dbias, accumulate=accumulate)


def profile_enable(on=True):
    lib().r3_profile_enable(C.c_int(1 if on else 0))


def profile_copy(dst, src):
    """Plain copy of src into dst by the library's calibration kernel."""
    assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
    _check(lib().r3_profile_copy(_p(dst), _p(src), C.c_size_t(src.numel() * src.element_size()), _stream()),
           "r3_profile_copy")


def profile_mfma(iters, random_operands, sink):
    """Launch the register-only MFMA loop; returns the FLOP it performs (the caller times it)."""
    _check(lib().r3_profile_mfma(C.c_int(iters), C.c_int(1 if random_operands else 0), _p(sink), _stream()),
           "r3_profile_mfma")
    return float(lib().r3_profile_mfma_flops(C.c_int(iters)))


def profile_gemm_mix(iters, src, sink, shape=0):
    """Launch the MFMA + LDS-read + global->LDS loop; src: 1 MiB of finite bf16 values on the device.
    shape 0: 8 waves of 128 x 64 (the kernels' shape); 1: 4 waves of 128 x 128."""
    assert src.numel() * src.element_size() >= 1 << 20
    _check(lib().r3_profile_gemm_mix(C.c_int(shape), C.c_int(iters), _p(src), _p(sink), _stream()),
           "r3_profile_gemm_mix")
    return float(lib().r3_profile_mfma_flops(C.c_int(iters)))


def profile_read():
    """{kernel name: (total milliseconds, launches)} recorded since profile_enable(True)."""
    out = {}
    for tag in range(lib().r3_profile_tags()):
        ms, n = C.c_double(0.0), C.c_int(0)
        _check(lib().r3_profile_read(tag, C.byref(ms), C.byref(n)), "r3_profile_read")
        if n.value:
            out[lib().r3_profile_name(tag).decode()] = (ms.value, n.value)
    return out
