"""The measurement aids of include/r3_profile.h (not part of the method): the per-launch timers see the
kernels of a forward pass and cost nothing when off, the copy kernel copies, the calibration loops run in both
tile shapes and report the FLOP they perform."""
import pytest
import torch

from paper_2510_11370_amd import r3, synth

pytestmark = pytest.mark.gpu


def test_launch_timers_see_the_forward_pass():
    sh = synth.LayerShape(T=300, d=256, E=128, K=8, F=256, sigma=0.02, seed=51)
    D = r3.desc(sh.T, sh.d, sh.E, sh.K, sh.F, sh.act)
    t = {k: synth.draw(sh, k, "cuda").to(torch.bfloat16) for k in ("x", "Wr", "Wg", "Wu", "Wd")}
    rec = torch.zeros(sh.T, sh.K, dtype=torch.uint8, device="cuda")
    buf = r3.LayerBuffers(D, backward=False, gathered_copy=False)
    r3.record_topk(D, t["x"].float() @ t["Wr"].float(), rec, buf.status)
    r3.profile_enable(True)
    for _ in range(3):
        r3.forward_one_call(buf, t["x"], t["Wr"], rec, t["Wg"], t["Wu"], t["Wd"])
    torch.cuda.synchronize()
    prof = r3.profile_read()
    r3.profile_enable(False)
    for name in ("replay_gate", "permute_index", "ffn1_swiglu", "ffn2_down", "combine"):
        ms, n = prof[name]
        assert n == 3 and 0.0 < ms < 1000.0, (name, ms, n)
    r3.forward_one_call(buf, t["x"], t["Wr"], rec, t["Wg"], t["Wu"], t["Wd"])   # timers off: nothing recorded
    torch.cuda.synchronize()
    r3.profile_enable(True)
    assert not r3.profile_read()
    r3.profile_enable(False)


def test_copy_and_calibration_kernels():
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    r3.profile_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    mix_src = torch.randn(1 << 19, device="cuda").to(torch.bfloat16)
    flop = r3.profile_mfma(100, True, sink)
    assert flop == r3.profile_mfma(100, False, sink) and flop > 0
    for shape in (0, 1):
        assert r3.profile_gemm_mix(100, mix_src, sink, shape=shape) == flop
    torch.cuda.synchronize()
    assert float(sink.item()) == 0.0
    with pytest.raises(r3.R3Error, match="INVALID_ARG"):
        r3.profile_gemm_mix(100, mix_src, sink, shape=2)
