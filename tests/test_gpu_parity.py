"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs.

Integer results (record, counts, offsets, permutations, copied rows) must match
bit for bit; floating point within the stated bars (tests/util.py).  Inputs of a
step come from the generator or from the oracle, never from another GPU call.
"""
import os

import numpy as np
import pytest
import torch

from oracle import sparse
from paper_2510_11370_amd import r3, synth
from util import Case, assert_close, assert_gates_close, dev, host, idx_dev, router_gradient_sigma

pytestmark = pytest.mark.gpu

SH = synth.LayerShape
# name -> shape.  "mfma" shapes satisfy the MFMA kernels' tiling (d, F multiples of 256,
# E multiple of 128); the others run the plain kernels.  Rows per expert span several
# 128-row tiles and leave ragged tails; some experts are empty.
SHAPES = {
    "config1_f32": synth.CONFIGS["tiny_f32"],
    "odd_f32": SH(T=37, d=50, E=5, K=3, F=30, act="f32", sigma=0.05, seed=21),
    "odd_bf16": SH(T=53, d=72, E=6, K=2, F=40, act="bf16", sigma=0.05, seed=22),
    "mfma_small": SH(T=300, d=256, E=128, K=8, F=256, act="bf16", sigma=0.02, seed=23),
    "mfma_ragged": SH(T=1111, d=512, E=128, K=8, F=768, act="bf16", sigma=0.02, zipf_s=1.2, seed=24),
    "mfma_fewexperts": SH(T=700, d=256, E=128, K=2, F=256, act="bf16", sigma=0.02, zipf_s=2.0, seed=25),
    # more than 256 experts: the record is uint16
    "mfma_u16": SH(T=900, d=256, E=384, K=4, F=256, act="bf16", sigma=0.02, zipf_s=1.0, seed=26),
    # other widths: 12 / 8 and 16 / 20 windows of 64 k in the row-tiled GEMMs, 3 / 4 and 2 / 5 column tiles
    "mfma_wide": SH(T=900, d=768, E=128, K=4, F=512, act="bf16", sigma=0.02, zipf_s=0.8, seed=27),
    "mfma_tall": SH(T=1500, d=1024, E=128, K=2, F=1280, act="bf16", sigma=0.02, seed=28),
    # a load so skewed that four experts hold nearly every token (about 9200 rows each): their
    # weight-gradient reductions are cut into five parts whose partial products are summed by a second launch
    "mfma_skewed": SH(T=9216, d=256, E=128, K=4, F=256, act="bf16", sigma=0.02, zipf_s=2.5, seed=29),
}


@pytest.fixture(autouse=True)
def _plain_env():
    os.environ.pop("R3_FORCE_SIMT", None)
    yield
    os.environ.pop("R3_FORCE_SIMT", None)


def sync():
    torch.cuda.synchronize()


# ------------------------------------------------------------------ record
@pytest.mark.parametrize("T,E,K,kind", [
    (256, 8, 2, "normal"), (4096, 128, 8, "normal"), (1000, 128, 8, "ties"), (333, 300, 4, "normal"),
    (100, 1024, 16, "normal"), (77, 128, 8, "nan"), (64, 64, 64, "normal"), (1, 128, 8, "normal"),
    (129, 512, 8, "ties"), (200, 40, 9, "ties"), (500, 256, 8, "ties"), (300, 64, 3, "ties"),
    (1000, 128, 5, "ties"), (77, 256, 8, "nan"), (4099, 128, 1, "normal"), (2048, 64, 8, "normal"),
])
def test_record_topk_bit_exact(T, E, K, kind):
    rng = np.random.default_rng(T * 1000 + E)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    if kind == "ties":
        lg = rng.integers(-2, 3, size=(T, E)).astype(np.float32)
        lg[lg == 0] = np.where(rng.random((lg == 0).sum()) < 0.5, 0.0, -0.0)
    if kind == "nan":
        lg[rng.random((T, E)) < 0.3] = np.nan
        lg[rng.random((T, E)) < 0.05] = np.inf
        lg[rng.random((T, E)) < 0.05] = -np.inf
        lg[0] = np.nan
    want = sparse.topk_mask(lg, K)
    D = r3.desc(T, 16, E, K, 16)
    out = torch.zeros(T, K, dtype=r3.idx_torch_dtype(D), device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    r3.record_topk(D, dev(lg, torch.float32), out, status)
    sync()
    got = out.cpu().numpy().astype(np.int32)
    assert np.array_equal(got, want)
    assert (int(status.item()) & r3.DATA_NONFINITE != 0) == (kind == "nan")


def test_record_topk_token_major_stride_and_leading_dim():
    T, E, K, L = 300, 128, 8, 3
    rng = np.random.default_rng(5)
    lg = rng.standard_normal((T, E + 16)).astype(np.float32)
    want = sparse.topk_mask(np.ascontiguousarray(lg[:, :E]), K)
    D = r3.desc(T, 16, E, K, 16, idx_token_stride=L * K)
    out = torch.full((T, L, K), 255, dtype=torch.uint8, device="cuda")
    r3.record_topk(D, dev(lg, torch.float32), out[:, 1], None)
    sync()
    got = out.cpu().numpy()
    assert np.array_equal(got[:, 1].astype(np.int32), want)
    assert (got[:, 0] == 255).all() and (got[:, 2] == 255).all()


# ------------------------------------------------------------------ permute
def _random_record(T, E, K, seed, skew=False):
    rng = np.random.default_rng(seed)
    p = None
    if skew:
        p = 1.0 / np.arange(1, E + 1) ** 1.5
        p /= p.sum()
    return np.stack([np.sort(rng.choice(E, K, replace=False, p=p)) for _ in range(T)]).astype(np.int32)


@pytest.mark.parametrize("T,E,K,d,act,skew", [
    (256, 8, 2, 128, "f32", False), (4096, 128, 8, 256, "bf16", False), (1, 128, 8, 64, "bf16", False),
    (100, 128, 8, 72, "bf16", True), (37, 5, 3, 50, "f32", False), (9000, 300, 4, 24, "bf16", True),
    (515, 16, 16, 33, "bf16", False),
])
def test_permute_bit_exact(T, E, K, d, act, skew):
    idx = _random_record(T, E, K, T + E, skew)
    x = synth._round(torch.randn(T, d, generator=torch.Generator().manual_seed(T)), act).numpy()
    counts, offsets, inv_perm, perm = sparse.permute(idx, E)
    Xp = sparse.gather_rows(x, perm, K)
    D = r3.desc(T, d, E, K, 16, act)
    adt = r3.act_dtype(D)
    S = T * K
    t = dict(counts=torch.empty(E, dtype=torch.int32, device="cuda"),
             offsets=torch.empty(E + 1, dtype=torch.int32, device="cuda"),
             inv_perm=torch.empty(S, dtype=torch.int32, device="cuda"),
             perm=torch.empty(S, dtype=torch.int32, device="cuda"),
             Xp=torch.empty(S, d, dtype=adt, device="cuda"))
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    r3.permute(D, dev(x, adt), idx_dev(idx, D), t["counts"], t["offsets"], t["inv_perm"], t["perm"], t["Xp"],
               r3.workspace(D, r3.OP_PERMUTE), status)
    sync()
    assert int(status.item()) == 0
    assert np.array_equal(t["counts"].cpu().numpy(), counts)
    assert np.array_equal(t["offsets"].cpu().numpy(), offsets)
    assert np.array_equal(t["inv_perm"].cpu().numpy(), inv_perm)
    assert np.array_equal(t["perm"].cpu().numpy(), perm)
    assert np.array_equal(host(t["Xp"]), Xp)  # rows are byte copies
    if skew and T < E:
        assert (counts == 0).any()  # empty experts are legal


def test_permute_flags_bad_record():
    T, E, K = 64, 16, 4
    idx = _random_record(T, E, K, 3)
    D = r3.desc(T, 16, E, K, 16)
    bufs = [torch.empty(n, dtype=torch.int32, device="cuda") for n in (E, E + 1, T * K, T * K)]
    for mutate, bit in ((lambda a: a.__setitem__((5, 2), 200), r3.DATA_IDX_RANGE),
                        (lambda a: a.__setitem__((7, 3), a[7, 0]), r3.DATA_IDX_DUP)):
        bad = idx.copy()
        mutate(bad)
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        r3.permute(D, None, idx_dev(bad, D), *bufs, None, r3.workspace(D, r3.OP_PERMUTE), status)
        sync()
        assert int(status.item()) & bit


# ------------------------------------------------------------------ gate
@pytest.mark.parametrize("name", ["config1_f32", "odd_f32", "odd_bf16", "mfma_small", "mfma_ragged", "mfma_u16"])
def test_replay_gate_and_logits(name):
    c = Case(SHAPES[name], backward=False)
    sh, D = c.shape, c.D
    g_ref = sparse.replay_gate(c.s, c.idx)
    gates = torch.empty(sh.T, sh.K, dtype=torch.float32, device="cuda")
    logits = torch.empty(sh.T, sh.E, dtype=torch.float32, device="cuda")
    agree = torch.zeros(2, dtype=torch.int64, device="cuda")
    r3.replay_gate(D, c.t["x"], c.t["Wr"], c.t["idx"], gates, bias=c.t["bias"], logits_out=logits,
                   agree_out=agree, ws=None)
    sync()
    lg = logits.cpu().numpy()
    assert np.abs(lg - c.s).max() <= 2e-5 * max(1.0, np.abs(c.s).max())
    assert_gates_close(gates.cpu().numpy(), g_ref)
    # agreement against the oracle's own top-K of the oracle's logits; a token whose K-th and
    # (K+1)-th logits are closer than the f32 accumulation error may legitimately differ
    own = sparse.topk_mask(c.s, sh.K)
    same, shared = sparse.agreement(own, c.idx)
    srt = np.sort(c.s, axis=1)
    near = int((srt[:, -sh.K] - srt[:, -sh.K - 1] < 1e-4).sum()) if sh.K < sh.E else 0
    assert abs(int(agree[0]) - same) <= near and abs(int(agree[1]) - shared) <= near
    # same call without logits_out (logits in the workspace) gives the same gates
    gates2 = torch.empty_like(gates)
    r3.replay_gate(D, c.t["x"], c.t["Wr"], c.t["idx"], gates2, bias=c.t["bias"],
                   ws=r3.workspace(D, r3.OP_REPLAY_GATE))
    sync()
    assert torch.equal(gates, gates2)


@pytest.mark.parametrize("E,d", [(128, 256), (16, 48)])       # the one-launch kernel; the plain kernels
def test_replay_gate_flags_bad_record_and_nonfinite_logits(E, d):
    T, K = 200, 4
    D = r3.desc(T, d, E, K, 256)
    g = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn(T, d, generator=g, device="cuda").to(torch.bfloat16)
    Wr = (torch.randn(d, E, generator=g, device="cuda") * d ** -0.5).to(torch.bfloat16)
    idx = _random_record(T, E, K, 9)
    gates = torch.empty(T, K, dtype=torch.float32, device="cuda")
    ws = r3.workspace(D, r3.OP_REPLAY_GATE)

    def status_after(xx, rec):
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        r3.replay_gate(D, xx, Wr, idx_dev(rec, D), gates, status=status, ws=ws)
        sync()
        return int(status.item())

    assert status_after(x, idx) == 0
    assert torch.isfinite(gates).all() and torch.allclose(gates.sum(dim=1), torch.ones(T, device="cuda"), atol=1e-5)
    bad = idx.copy()
    bad[17, 1] = 250                                   # an expert id >= E
    assert status_after(x, bad) == r3.DATA_IDX_RANGE
    xn = x.clone()
    xn[33, 7] = float("inf")                           # every logit of token 33 is inf or NaN
    assert status_after(xn, idx) == r3.DATA_NONFINITE


def test_recompute_routing_replay_is_plain_topk_gating():
    """The variant that records from the training engine's own logits (Related Works, "Routing Replay"):
    r3_record_topk on the layer's training logits, replayed into the same layer.  With an unchanged model
    (mini step 1) the replay changes nothing: every token agrees, and the gates are the standard
    top-K softmax gates (third equation of Section 4.1 = its replay-gate equation with I_infer = I_train)."""
    c = Case(SHAPES["mfma_small"], backward=False)
    sh, D = c.shape, c.D
    gates = torch.empty(sh.T, sh.K, dtype=torch.float32, device="cuda")
    logits = torch.empty(sh.T, sh.E, dtype=torch.float32, device="cuda")
    rec = torch.zeros(sh.T, sh.K, dtype=r3.idx_torch_dtype(D), device="cuda")
    ws = r3.workspace(D, r3.OP_REPLAY_GATE)
    r3.replay_gate(D, c.t["x"], c.t["Wr"], rec, gates, logits_out=logits, ws=ws)       # training logits
    r3.record_topk(D, logits, rec, None)                                               # recompute-stage record
    agree = torch.zeros(2, dtype=torch.int64, device="cuda")
    r3.replay_gate(D, c.t["x"], c.t["Wr"], rec, gates, agree_out=agree, ws=ws)         # update-stage replay
    sync()
    assert (int(agree[0]), int(agree[1])) == (sh.T, sh.T * sh.K)
    lg = logits.cpu().numpy()
    own = sparse.topk_mask(lg, sh.K)
    assert np.array_equal(rec.cpu().numpy().astype(np.int32), own)
    # standard gating from a library softmax over all experts, renormalised over the top-K set
    p = torch.softmax(torch.from_numpy(lg.astype(np.float64)), dim=1).numpy()
    sel = np.take_along_axis(p, own, axis=1)
    assert_gates_close(gates.cpu().numpy(), sel / sel.sum(axis=1, keepdims=True))


# ------------------------------------------------------------------ expert FFN and combine, step by step
@pytest.mark.parametrize("name,simt", [("config1_f32", False), ("odd_bf16", False), ("mfma_small", False),
                                       ("mfma_ragged", False), ("mfma_fewexperts", False),
                                       ("mfma_small", True)])
def test_grouped_ffn_and_combine_steps(name, simt):
    if simt:
        os.environ["R3_FORCE_SIMT"] = "1"
    c = Case(SHAPES[name], backward=False, scale_w=5.0)
    sh, D, n = c.shape, c.D, c.np
    adt = r3.act_dtype(D)
    counts, offsets, inv_perm, perm = sparse.permute(c.idx, sh.E)
    Xp = sparse.gather_rows(n["x"], perm, sh.K)
    a, b, h, o = sparse.grouped_ffn(Xp, offsets, n["Wg"], n["Wu"], n["Wd"])
    S = sh.T * sh.K
    Yp, H, A, B = (torch.zeros(S, w, dtype=adt, device="cuda") for w in (sh.d, sh.F, sh.F, sh.F))
    r3.grouped_ffn(D, dev(Xp, adt), dev(offsets, torch.int32), c.t["Wg"], c.t["Wu"], c.t["Wd"], Yp, H, A, B,
                   ws=r3.workspace(D, r3.OP_GROUPED_FFN))
    sync()
    # what the call saves for the backward are the two factors of the SwiGLU backward, derived here from
    # the oracle's pre-activations: FA = b silu'(a) (dA = dh FA), FB = silu(a) (dB = dh FB)
    sg = 1.0 / (1.0 + np.exp(-a))
    assert_close(host(A), b * sg * (1.0 + a * (1.0 - sg)), "FA = b silu'(a)", c.rel)
    assert_close(host(B), a * sg, "FB = silu(a)", c.rel)
    assert_close(host(H), h, "H", c.rel)
    assert_close(host(Yp), o, "Yp", c.rel)
    # the same call reading the token rows through perm instead of a gathered copy: the gather moves
    # bytes, so every output must be bit-identical
    Yp2, H2, A2, B2 = (torch.zeros(S, w, dtype=adt, device="cuda") for w in (sh.d, sh.F, sh.F, sh.F))
    r3.grouped_ffn(D, None, dev(offsets, torch.int32), c.t["Wg"], c.t["Wu"], c.t["Wd"], Yp2, H2, A2, B2,
                   ws=r3.workspace(D, r3.OP_GROUPED_FFN), x=c.t["x"], perm=dev(perm, torch.int32))
    sync()
    for got, want, nm in ((Yp2, Yp, "Yp"), (H2, H, "H"), (A2, A, "A"), (B2, B, "B")):
        assert torch.equal(got, want), nm
    # combine on oracle-made inputs: o rounded to the activation dtype, oracle gates as f32
    g = sparse.replay_gate(c.s, c.idx)
    o_act = synth._round(torch.from_numpy(o).float(), sh.act).numpy()
    y_ref = sparse.combine(o_act.astype(np.float64), g.astype(np.float32).astype(np.float64), inv_perm)
    y = torch.empty(sh.T, sh.d, dtype=adt, device="cuda")
    r3.combine(D, dev(o_act, adt), dev(g, torch.float32), dev(inv_perm, torch.int32), y)
    sync()
    assert_close(host(y), y_ref, "y", 4e-3 if sh.act == "bf16" else 1e-5)


# ------------------------------------------------------------------ whole forward and backward
def _run_forward(c, backward):
    buf = r3.LayerBuffers(c.D, backward=backward)
    r3.forward(buf, c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], bias=c.t["bias"])
    sync()
    return buf


@pytest.mark.parametrize("name,simt", [("config1_f32", False), ("odd_f32", False), ("odd_bf16", False),
                                       ("mfma_small", False), ("mfma_ragged", False), ("mfma_ragged", True),
                                       ("mfma_u16", False)])
def test_forward_chain(name, simt):
    if simt:
        os.environ["R3_FORCE_SIMT"] = "1"
    c = Case(SHAPES[name], backward=False, scale_w=5.0)
    n = c.np
    ref = sparse.forward(n["x"], n["Wr"], c.idx, n["Wg"], n["Wu"], n["Wd"], n["bias"])
    buf = _run_forward(c, backward=False)
    assert int(buf.status.item()) == 0
    for k in ("counts", "offsets", "inv_perm", "perm"):
        assert np.array_equal(getattr(buf, k).cpu().numpy(), ref[k]), k
    assert np.array_equal(host(buf.Xp), ref["Xp"])
    assert_gates_close(buf.gates.cpu().numpy(), ref["g"])
    assert_close(host(buf.y), ref["y"], "y", c.rel)
    # recompute stage and update stage run the same kernels: bit-identical forward, twice
    buf2 = _run_forward(c, backward=True)
    assert torch.equal(buf.y, buf2.y) and torch.equal(buf.gates, buf2.gates)
    # forward without the gathered copy of the tokens (rows read through perm in the expert GEMM)
    buf3 = r3.LayerBuffers(c.D, backward=False, gathered_copy=False)
    r3.forward(buf3, c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], bias=c.t["bias"])
    sync()
    assert buf3.Xp is None and torch.equal(buf.y, buf3.y) and torch.equal(buf.Yp, buf3.Yp)


@pytest.mark.parametrize("name,simt", [("config1_f32", False), ("odd_f32", False), ("odd_bf16", False),
                                       ("mfma_small", False), ("mfma_ragged", False),
                                       ("mfma_fewexperts", False), ("mfma_small", True), ("mfma_u16", False), ("mfma_u16", True),
                                       ("mfma_wide", False), ("mfma_tall", False), ("mfma_skewed", False)])
def test_backward_chain(name, simt):
    if simt:
        os.environ["R3_FORCE_SIMT"] = "1"
    c = Case(SHAPES[name], backward=True, scale_w=5.0)
    n, sh = c.np, c.shape
    fwd = sparse.forward(n["x"], n["Wr"], c.idx, n["Wg"], n["Wu"], n["Wd"], n["bias"])
    ref = sparse.backward(n["dy"], n["x"], n["Wr"], c.idx, n["Wg"], n["Wu"], n["Wd"], fwd, want_dbias=True)
    buf = _run_forward(c, backward=True)
    dbias = torch.zeros(sh.E, dtype=torch.float32, device="cuda")
    r3.backward(buf, c.t["dy"], c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], dbias=dbias)
    sync()
    assert_close(host(buf.dx), ref["dx"], "dx", c.rel)
    sig_w, sig_b = (None, None) if sh.act == "f32" else router_gradient_sigma(n["x"], n["dy"], c.idx, fwd, sh.E)
    assert_close(buf.dW_r.cpu().numpy(), ref["dWr"], "dW_r", c.rel, sig_w)
    assert_close(dbias.cpu().numpy(), ref["dbias"], "dbias", c.rel, sig_b)
    for got, key in ((buf.dW_gate, "dWg"), (buf.dW_up, "dWu"), (buf.dW_down, "dWd")):
        got = got.cpu().numpy()
        for e in range(sh.E):  # per expert tensor, norm-wise; empty experts must be exactly zero
            if fwd["counts"][e] == 0:
                assert not got[e].any(), (key, e)
            else:
                nr = np.linalg.norm(ref[key][e])
                assert np.linalg.norm(got[e] - ref[key][e]) <= c.rel * nr + 1e-30, (key, e)
    # accumulate=1 adds the same gradient once more; a second identical call is bit-identical
    keep = {k: getattr(buf, k).clone() for k in ("dx", "dW_r", "dW_gate", "dW_up", "dW_down")}
    r3.backward(buf, c.t["dy"], c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"])
    sync()
    for k, v in keep.items():
        assert torch.equal(getattr(buf, k), v), k
    r3.backward(buf, c.t["dy"], c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"],
                accumulate=True)
    sync()
    for k in ("dW_r", "dW_gate", "dW_up", "dW_down"):
        assert torch.allclose(getattr(buf, k), 2 * keep[k], rtol=1e-5, atol=1e-6 * float(keep[k].abs().max())), k
    # without the gathered copy of the tokens: forward and backward read x through perm (inside the expert
    # GEMMs' tile loads, or row by row in the plain kernels); every result is the same bit for bit
    buf2 = r3.LayerBuffers(c.D, backward=True, gathered_copy=False)
    r3.forward(buf2, c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], bias=c.t["bias"])
    r3.backward(buf2, c.t["dy"], c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"])
    sync()
    assert buf2.Xp is None and int(buf2.status.item()) == 0
    for k, v in keep.items():
        assert torch.equal(getattr(buf2, k), v), k


@pytest.mark.parametrize("name,simt", [("config1_f32", False), ("odd_bf16", False), ("mfma_small", False),
                                       ("mfma_ragged", False), ("mfma_fewexperts", False), ("mfma_small", True),
                                       ("mfma_u16", False), ("mfma_wide", False), ("mfma_tall", False),
                                       ("mfma_skewed", False)])
def test_one_call_forward_and_its_backward(name, simt):
    """r3_moe_forward (gate folded into the expert network: H and Yp come out gate-scaled, the combination
    is a plain sum) and r3_moe_backward told so, against the oracle's forward and backward."""
    if simt:
        os.environ["R3_FORCE_SIMT"] = "1"
    c = Case(SHAPES[name], backward=True, scale_w=5.0)
    n, sh = c.np, c.shape
    fwd = sparse.forward(n["x"], n["Wr"], c.idx, n["Wg"], n["Wu"], n["Wd"], n["bias"])
    ref = sparse.backward(n["dy"], n["x"], n["Wr"], c.idx, n["Wg"], n["Wu"], n["Wd"], fwd, want_dbias=True)
    buf = r3.LayerBuffers(c.D, backward=True, gathered_copy=False)
    agree = torch.zeros(2, dtype=torch.int64, device="cuda")
    r3.forward_one_call(buf, c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], bias=c.t["bias"],
                        agree_out=agree)
    sync()
    assert int(buf.status.item()) == 0
    for k in ("counts", "offsets", "inv_perm", "perm"):
        assert np.array_equal(getattr(buf, k).cpu().numpy(), fwd[k]), k
    assert_gates_close(buf.gates.cpu().numpy(), fwd["g"])
    grow = fwd["g"].reshape(-1)[fwd["perm"]]                       # the gate of every expert-sorted row
    assert_close(host(buf.H), grow[:, None] * fwd["h"], "g*H", c.rel)
    assert_close(host(buf.Yp), grow[:, None] * fwd["o"], "g*o", c.rel)
    assert_close(host(buf.y), fwd["y"], "y", c.rel)
    assert 0 < int(agree[0]) <= sh.T and int(agree[1]) <= sh.T * sh.K
    if name == "mfma_skewed":
        assert fwd["counts"].max() > 8192      # (what makes the backward split its reductions)
    dbias = torch.zeros(sh.E, dtype=torch.float32, device="cuda")
    r3.backward(buf, c.t["dy"], c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], dbias=dbias)
    sync()
    assert buf.gated
    assert_close(host(buf.dx), ref["dx"], "dx", c.rel)
    sig_w, sig_b = (None, None) if sh.act == "f32" else router_gradient_sigma(n["x"], n["dy"], c.idx, fwd, sh.E)
    assert_close(buf.dW_r.cpu().numpy(), ref["dWr"], "dW_r", c.rel, sig_w)
    assert_close(dbias.cpu().numpy(), ref["dbias"], "dbias", c.rel, sig_b)
    for got, key in ((buf.dW_gate, "dWg"), (buf.dW_up, "dWu"), (buf.dW_down, "dWd")):
        got = got.cpu().numpy()
        for e in range(sh.E):
            if fwd["counts"][e] == 0:
                assert not got[e].any(), (key, e)
            else:   # per expert tensor, norm-wise (an expert with two or three rows has no element scale)
                nr = np.linalg.norm(ref[key][e])
                assert np.linalg.norm(got[e] - ref[key][e]) <= c.rel * nr + 1e-30, (key, e)
    # a second pass over the same buffers is bit-identical
    keep = {k: getattr(buf, k).clone() for k in ("y", "dx", "dW_r", "dW_gate", "dW_up", "dW_down")}
    r3.forward_one_call(buf, c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], bias=c.t["bias"])
    r3.backward(buf, c.t["dy"], c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"])
    sync()
    for k, v in keep.items():
        assert torch.equal(getattr(buf, k), v), k


def test_router_gradient_is_zero_off_the_replayed_set():
    """An expert in the training top-K that was not replayed gets no gradient from that token."""
    sh = SH(T=64, d=128, E=8, K=2, F=256, act="f32", sigma=0.5, seed=31)
    c = Case(sh, backward=True, scale_w=5.0)
    own = sparse.topk_mask(c.s, sh.K)
    assert (own != c.idx).any()
    buf = _run_forward(c, backward=True)
    dbias = torch.zeros(sh.E, dtype=torch.float32, device="cuda")
    # single-token probe: zero every dy row but one whose record differs from its own top-K
    t = int(np.nonzero((own != c.idx).any(1))[0][0])
    dy = torch.zeros_like(c.t["dy"])
    dy[t] = c.t["dy"][t]
    r3.backward(buf, dy, c.t["x"], c.t["Wr"], c.t["idx"], c.t["Wg"], c.t["Wu"], c.t["Wd"], dbias=dbias)
    sync()
    db = dbias.cpu().numpy()
    on = np.zeros(sh.E, bool)
    on[c.idx[t]] = True
    assert np.all(db[~on] == 0.0) and np.all(db[on] != 0.0)
    assert abs(db.sum()) <= 1e-5 * np.abs(db).max()


# ------------------------------------------------------------------ host-side error handling
def test_host_errors_are_returned_before_launch():
    D = r3.desc(16, 16, 8, 2, 16, "f32")
    x = torch.zeros(16, 16, device="cuda")
    with pytest.raises(r3.R3Error, match="INVALID_ARG"):
        r3.combine(D, None, x, x, x)
    with pytest.raises(r3.R3Error, match="INVALID_ARG"):
        r3.combine(r3.desc(16, 16, 8, 9, 16, "f32"), x, x, x, x)  # K > E
    with pytest.raises(r3.R3Error, match="UNSUPPORTED"):
        r3.combine(r3.desc(16, 16, 300, 2, 16, "f32", idx_dtype=torch.uint8), x, x, x, x)
    with pytest.raises(r3.R3Error, match="WORKSPACE"):
        r3.permute(D, x, x, x, x, x, x, x, torch.empty(0, dtype=torch.uint8, device="cuda"))
    with pytest.raises(r3.R3Error, match="INVALID_ARG"):
        r3.combine(D, x.view(-1)[1:], x, x, x)  # misaligned
    with pytest.raises(r3.R3Error, match="INVALID_ARG"):
        r3.grouped_ffn(D, None, x, x, x, x, x, x, x=x)  # neither Xp nor (x, perm)
