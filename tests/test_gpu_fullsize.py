"""Parity at the full size of the forward+backward single-layer configuration (T=16384, d=2048, E=128, K=8,
F=768, bf16) in the launch configuration bench.py times.  The oracle runs the whole layer once, forward and
backward over all 16384 tokens (about half a minute on 16 cores, 20 GB of float64), and every output is
compared element by element: record, permutation, gates, H, Yp, y, dx, dW_r under the full upstream gradient
and the three weight gradients of all 128 experts."""
import numpy as np
import pytest
import torch

from oracle import sparse
from paper_2510_11370_amd import r3, synth
from util import assert_close, assert_gates_close, host, router_gradient_sigma

pytestmark = pytest.mark.gpu

SHAPE = synth.CONFIGS["fwdbwd_16k"]


@pytest.fixture(scope="module")
def full():
    sh = SHAPE
    dev = "cuda"
    D = r3.desc(sh.T, sh.d, sh.E, sh.K, sh.F, sh.act)
    # same bytes on both sides: drawn once (on the GPU, it is only a generator), rounded to bf16
    t = {k: synth.draw(sh, k, dev).to(torch.bfloat16) for k in ("x", "Wr", "Wg", "Wu", "Wd", "dy")}
    n = {k: t[k].float().cpu().numpy() for k in ("x", "Wr", "dy")}
    noise = synth.draw(sh, "noise", "cpu").numpy()
    s = sparse.router_logits(n["x"], n["Wr"])                       # oracle training logits, all tokens
    s_infer = (s + noise).astype(np.float32)
    idx = sparse.topk_mask(s_infer, sh.K)                            # oracle record
    # GPU record from the same inference-logit bytes
    rec = torch.zeros(sh.T, sh.K, dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    r3.record_topk(D, torch.from_numpy(s_infer).to(dev), rec, status)
    buf = r3.LayerBuffers(D, backward=True)
    r3.forward(buf, t["x"], t["Wr"], rec, t["Wg"], t["Wu"], t["Wd"])
    r3.backward(buf, t["dy"], t["x"], t["Wr"], rec, t["Wg"], t["Wu"], t["Wd"])
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and int(buf.status.item()) == 0
    return dict(sh=sh, D=D, t=t, n=n, s=s, idx=idx, rec=rec, buf=buf)


@pytest.fixture(scope="module")
def ref(full):
    """The oracle's forward and backward over all tokens (same input bytes as the GPU run)."""
    n = full["n"]
    Wg, Wu, Wd = _weights_of(full, slice(None))
    fwd = sparse.forward(n["x"], n["Wr"], full["idx"], Wg, Wu, Wd)
    bwd = sparse.backward(n["dy"], n["x"], n["Wr"], full["idx"], Wg, Wu, Wd, fwd)
    for k in ("Xp", "a", "b", "s"):          # not compared below; frees 4 GB
        fwd.pop(k)
    for k in ("dO", "da", "db", "dXp", "dxr", "ds"):
        bwd.pop(k)
    return fwd, bwd


def _weights_of(full, experts):
    t = full["t"]
    return tuple(t[k][experts].float().cpu().numpy() for k in ("Wg", "Wu", "Wd"))


def test_record_and_permutation_bit_exact(full):
    sh, buf = full["sh"], full["buf"]
    assert np.array_equal(full["rec"].cpu().numpy().astype(np.int32), full["idx"])
    counts, offsets, inv_perm, perm = sparse.permute(full["idx"], sh.E)
    assert np.array_equal(buf.counts.cpu().numpy(), counts)
    assert np.array_equal(buf.offsets.cpu().numpy(), offsets)
    assert np.array_equal(buf.inv_perm.cpu().numpy(), inv_perm)
    assert np.array_equal(buf.perm.cpu().numpy(), perm)
    rows = np.random.default_rng(0).choice(sh.T * sh.K, 4096, replace=False)
    got = host(buf.Xp[torch.from_numpy(rows).cuda()])
    assert np.array_equal(got, full["n"]["x"][perm[rows] // sh.K])


def test_gates_all_tokens(full):
    assert_gates_close(full["buf"].gates.cpu().numpy(), sparse.replay_gate(full["s"], full["idx"]))


def test_forward_every_row_and_token(full, ref):
    buf, (fwd, _) = full["buf"], ref
    assert_close(host(buf.H), fwd["h"], "H (all rows)", 1e-2)
    assert_close(host(buf.Yp), fwd["o"], "Yp (all rows)", 1e-2)
    assert_close(host(buf.y), fwd["y"], "y (all tokens)", 1e-2)


def test_input_gradient_every_token(full, ref):
    assert_close(host(full["buf"].dx), ref[1]["dx"], "dx (all tokens)", 1e-2)


def test_router_weight_gradient_under_the_full_upstream_gradient(full, ref):
    sh, buf, n = full["sh"], full["buf"], full["n"]
    fwd, bwd = ref
    sig, _ = router_gradient_sigma(n["x"], n["dy"], full["idx"], fwd, sh.E)
    assert_close(buf.dW_r.cpu().numpy(), bwd["dWr"], "dW_r (dense dy)", 1e-2, sigma=sig)


def test_expert_weight_gradients_all_experts(full, ref):
    sh, buf = full["sh"], full["buf"]
    _, bwd = ref
    for got, want, name in ((buf.dW_gate, bwd["dWg"], "dW_gate"), (buf.dW_up, bwd["dWu"], "dW_up"),
                            (buf.dW_down, bwd["dWd"], "dW_down")):
        for e0 in range(0, sh.E, 16):        # 16 experts at a time: bounded host memory for the differences
            g = got[e0:e0 + 16].cpu().numpy()
            for e in range(e0, min(e0 + 16, sh.E)):
                assert_close(g[e - e0], want[e], "%s[%d]" % (name, e), 1e-2)


def test_router_weight_gradient_with_sparse_upstream_gradient(full):
    """dW_r sums over every token; with dy zero outside a sample the oracle needs only the sample."""
    sh, t, n = full["sh"], full["t"], full["n"]
    tok = np.sort(np.random.default_rng(2).choice(sh.T, 96, replace=False))
    dy = torch.zeros_like(t["dy"])
    sel = torch.from_numpy(tok).cuda()
    dy[sel] = t["dy"][sel]
    keep = full["buf"].dW_r
    buf = r3.LayerBuffers(full["D"], backward=True)       # its own buffers: the module's results stay as they are
    r3.forward(buf, t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    r3.backward(buf, dy, t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    torch.cuda.synchronize()
    Wg, Wu, Wd = _weights_of(full, slice(None))
    fwd = sparse.forward(n["x"][tok], n["Wr"], full["idx"][tok], Wg, Wu, Wd)
    _, _, ds = sparse.gate_backward(n["dy"][tok], fwd["o"], fwd["g"], full["idx"][tok], fwd["inv_perm"], sh.E)
    dWr = n["x"][tok].astype(np.float64).T @ ds
    assert_close(buf.dW_r.cpu().numpy(), dWr, "dW_r(sparse dy)", 1e-2)
    other = np.setdiff1d(np.arange(sh.T), tok)[:512]
    assert not buf.dx[torch.from_numpy(other).cuda()].any()  # no gradient where dy is zero
    assert not torch.equal(keep, buf.dW_r)


def test_without_the_gathered_copy_bit_identical(full):
    """The launch configuration bench.py times: no expert-sorted copy of the tokens; forward and backward read
    x through the permutation inside the expert GEMMs.  Every output equals the gathered-copy path's bit for bit."""
    sh, t, buf = full["sh"], full["t"], full["buf"]
    buf2 = r3.LayerBuffers(full["D"], backward=True, gathered_copy=False)
    r3.forward(buf2, t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    r3.backward(buf2, t["dy"], t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    torch.cuda.synchronize()
    assert buf2.Xp is None and int(buf2.status.item()) == 0
    for k in ("y", "Yp", "H", "gates", "dx", "dW_r", "dW_gate", "dW_up", "dW_down"):
        assert torch.equal(getattr(buf, k), getattr(buf2, k)), k


def test_bench_configuration_one_call_forward_and_gated_backward(full, ref):
    """Exactly what bench.py launches: r3_moe_forward (one call, no expert-sorted copy, the gate folded into H
    and Yp) and r3_moe_backward told so.  Every output against the oracle: H and Yp as g*h and g*o on every row,
    y and dx on every token, dW_r under the full upstream gradient, all 128 experts' weight gradients."""
    sh, t, n = full["sh"], full["t"], full["n"]
    fwd, bwd = ref
    buf = r3.LayerBuffers(full["D"], backward=True, gathered_copy=False)
    r3.forward_one_call(buf, t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    r3.backward(buf, t["dy"], t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    torch.cuda.synchronize()
    assert buf.gated and buf.Xp is None and int(buf.status.item()) == 0
    for k in ("counts", "offsets", "inv_perm", "perm"):
        assert torch.equal(getattr(buf, k), getattr(full["buf"], k)), k
    assert_gates_close(buf.gates.cpu().numpy(), fwd["g"])
    grow = fwd["g"].reshape(-1)[fwd["perm"]]
    assert_close(host(buf.H), grow[:, None] * fwd["h"], "g*H (all rows, one call)", 1e-2)
    assert_close(host(buf.Yp), grow[:, None] * fwd["o"], "g*Yp (all rows, one call)", 1e-2)
    assert_close(host(buf.y), fwd["y"], "y (all tokens, one call)", 1e-2)
    assert_close(host(buf.dx), bwd["dx"], "dx (all tokens, one call)", 1e-2)
    sig, _ = router_gradient_sigma(n["x"], n["dy"], full["idx"], fwd, sh.E)
    assert_close(buf.dW_r.cpu().numpy(), bwd["dWr"], "dW_r (dense dy, one call)", 1e-2, sigma=sig)
    for got, want, name in ((buf.dW_gate, bwd["dWg"], "dW_gate"), (buf.dW_up, bwd["dWu"], "dW_up"),
                            (buf.dW_down, bwd["dWd"], "dW_down")):
        for e0 in range(0, sh.E, 16):
            g = got[e0:e0 + 16].cpu().numpy()
            for e in range(e0, min(e0 + 16, sh.E)):
                assert_close(g[e - e0], want[e], "%s[%d] (one call)" % (name, e), 1e-2)
