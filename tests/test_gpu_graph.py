"""The library allocates nothing, never synchronises and records no memset, so a caller may capture its calls in a
HIP graph.  Checked here: record + forward + backward captured once, replayed several times with eager work
and synchronisations between the replays, every replay bit-identical to the eager result."""
import pytest
import torch

from paper_2510_11370_amd import r3, synth

pytestmark = pytest.mark.gpu


# (gathered copy of the tokens, forward as one call); the middle case is what bench.py launches, the skewed one
# also splits weight-gradient reductions (partial products summed by a second launch)
@pytest.mark.parametrize("gathered_copy,one_call,skewed", [(False, False, False), (False, True, False),
                                                           (True, False, False), (False, True, True)])
def test_forward_backward_replays_from_a_graph(gathered_copy, one_call, skewed):
    sh = synth.LayerShape(T=1111, d=512, E=128, K=8, F=768, sigma=0.02, zipf_s=1.2, seed=41)
    if skewed:
        sh = synth.LayerShape(T=9216, d=256, E=128, K=4, F=256, sigma=0.02, zipf_s=2.5, seed=42)
    dev = "cuda"
    D = r3.desc(sh.T, sh.d, sh.E, sh.K, sh.F, sh.act)
    t = {k: synth.draw(sh, k, dev).to(torch.bfloat16) for k in ("x", "Wr", "Wg", "Wu", "Wd", "dy")}
    bias = synth.draw(sh, "bias", dev)
    logits = (t["x"].float() @ t["Wr"].float()) + bias + synth.draw(sh, "noise", dev)
    rec = torch.zeros(sh.T, sh.K, dtype=torch.uint8, device=dev)
    buf = r3.LayerBuffers(D, backward=True, gathered_copy=gathered_copy)
    outs = ("y", "dx", "dW_r", "dW_gate", "dW_up", "dW_down", "gates", "perm")

    def step():
        r3.record_topk(D, logits, rec, buf.status)
        (r3.forward_one_call if one_call else r3.forward)(buf, t["x"], t["Wr"], rec, t["Wg"], t["Wu"], t["Wd"],
                                                          bias=bias)
        r3.backward(buf, t["dy"], t["x"], t["Wr"], rec, t["Wg"], t["Wu"], t["Wd"])

    step()
    torch.cuda.synchronize()
    eager = {k: getattr(buf, k).clone() for k in outs}
    eager_rec = rec.clone()

    side = torch.cuda.Stream()           # capture on a side stream (default priority), as torch asks
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                           # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for replay in range(4):
        # eager work and a synchronisation between replays; the outputs are wiped so that a replay that did
        # nothing, or only part of its work, cannot pass
        for k in outs:
            getattr(buf, k).zero_()
        rec.zero_()
        scratch = torch.randn(1 << 20, device=dev).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(scratch)
        assert torch.equal(rec, eager_rec), replay
        for k in outs:
            assert torch.equal(getattr(buf, k), eager[k]), (k, replay)
    assert int(buf.status.item()) == 0
