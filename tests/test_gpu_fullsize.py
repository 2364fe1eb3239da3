"""Parity at the benchmark's full size and launch configuration (T=16384, d=2048, E=128, K=8, F=768, bf16,
forward + backward), on outputs the oracle can compute one by one: every integer result in full, all gates,
and sampled tokens / experts for the floating-point tensors.  Token-wise outputs (y, dx) depend only on their
own token, so the oracle runs the sampled tokens as a small batch of its own; an expert's weight gradients
need only that expert's rows."""
import numpy as np
import pytest
import torch

from oracle import sparse
from paper_2510_11370_amd import r3, synth
from util import assert_close, assert_gates_close, host

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


def test_sampled_tokens_forward_and_dx(full):
    sh, buf, n = full["sh"], full["buf"], full["n"]
    tok = np.sort(np.random.default_rng(1).choice(sh.T, 48, replace=False))
    Wg, Wu, Wd = _weights_of(full, slice(None))
    Wr = n["Wr"]
    fwd = sparse.forward(n["x"][tok], Wr, full["idx"][tok], Wg, Wu, Wd)
    assert_close(host(buf.y[torch.from_numpy(tok).cuda()]), fwd["y"], "y[sample]", 1e-2)
    # dx of a token needs only that token; the weight gradients of this small batch are not compared
    bwd = sparse.backward(n["dy"][tok], n["x"][tok], Wr, full["idx"][tok], Wg, Wu, Wd, fwd)
    dx = bwd["dx"]
    assert_close(host(buf.dx[torch.from_numpy(tok).cuda()]), dx, "dx[sample]", 1e-2)


@pytest.mark.parametrize("which", ["most_loaded", "least_loaded", "seeded"])
def test_expert_weight_gradients(full, which):
    sh, buf, n = full["sh"], full["buf"], full["n"]
    counts, offsets, inv_perm, perm = sparse.permute(full["idx"], sh.E)
    e = {"most_loaded": int(np.argmax(counts)), "least_loaded": int(np.argmin(counts)), "seeded": 77}[which]
    r0, r1 = int(offsets[e]), int(offsets[e + 1])
    slots = perm[r0:r1]
    tok, j = slots // sh.K, slots % sh.K
    Xp = n["x"][tok]
    Wg, Wu, Wd = _weights_of(full, slice(e, e + 1))
    off1 = np.array([0, r1 - r0], np.int32)
    a, b, h, o = sparse.grouped_ffn(Xp, off1, Wg, Wu, Wd)
    g = sparse.replay_gate(full["s"][tok], full["idx"][tok])[np.arange(len(tok)), j]
    dO = g[:, None] * n["dy"][tok].astype(np.float64)
    _, _, _, dWg, dWu, dWd = sparse.grouped_ffn_backward(Xp, off1, Wg, Wu, Wd, a, b, h, dO)
    # forward tensors of that expert's rows, while we have them
    assert_close(host(buf.Yp[r0:r1]), o, "Yp[e]", 1e-2)
    assert_close(host(buf.H[r0:r1]), h, "H[e]", 1e-2)
    for got, ref, name in ((buf.dW_gate[e], dWg[0], "dW_gate"), (buf.dW_up[e], dWu[0], "dW_up"),
                           (buf.dW_down[e], dWd[0], "dW_down")):
        assert_close(got.cpu().numpy(), ref, "%s[%d]" % (name, e), 1e-2)


def test_router_weight_gradient_with_sparse_upstream_gradient(full):
    """dW_r sums over every token; with dy zero outside a sample the oracle needs only the sample."""
    sh, buf, t, n = full["sh"], full["buf"], full["t"], full["n"]
    tok = np.sort(np.random.default_rng(2).choice(sh.T, 96, replace=False))
    dy = torch.zeros_like(t["dy"])
    sel = torch.from_numpy(tok).cuda()
    dy[sel] = t["dy"][sel]
    keep = buf.dW_r.clone()
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
    r3.backward(buf, t["dy"], t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])   # (an earlier test used a sparse dy)
    buf2 = r3.LayerBuffers(full["D"], backward=True, gathered_copy=False)
    r3.forward(buf2, t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    r3.backward(buf2, t["dy"], t["x"], t["Wr"], full["rec"], t["Wg"], t["Wu"], t["Wd"])
    torch.cuda.synchronize()
    assert buf2.Xp is None and int(buf2.status.item()) == 0
    for k in ("y", "Yp", "H", "gates", "dx", "dW_r", "dW_gate", "dW_up", "dW_down"):
        assert torch.equal(getattr(buf, k), getattr(buf2, k)), k
