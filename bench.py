#!/usr/bin/env python3
"""Throughput of the replayed MoE layer (record + replay gate + permute + grouped SwiGLU FFN +
combine + backward) on one MI355X, with the dominant kernel's roofline and the CPU oracle beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload zipf_64k]

One step = one pass of the whole hot path over one batch of seeded synthetic input that is
already resident in HBM:  r3_record_topk (inference logits -> record), the replayed forward
(r3_moe_forward: gate, dispatch, grouped SwiGLU FFN, combination; --six-calls runs the same steps as
r3_replay_gate, r3_permute, r3_grouped_ffn, r3_combine), r3_moe_backward.  Prints ONE JSON line.

The default line is the largest forward+backward configuration (zipf_64k: T=65536, load skewed by a
Zipf router bias); the 16384-token forward+backward configuration is timed in the same run, K steps
after W warm-up steps of its own, and reported under "also": {"fwdbwd_16k": ...} with its own kernel
table and roofline.  --workload NAME times that configuration alone.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published


def kernel_work(sh, idx_bytes=1):
    """Algorithmic work of one launch of each timed kernel: (kind, flops or bytes)."""
    T, d, E, K, F = sh.T, sh.d, sh.E, sh.K, sh.F
    S = T * K
    eb = 2  # bf16
    nparts = 2 * (F // 256)   # partial dot products per row left by the down projection's gradient GEMM
    return {
        "record_topk": ("hbm", T * (E * 4 + K * idx_bytes)),
        "agreement": ("hbm", T * (E * 4 + K * idx_bytes)),
        "router_logits": ("hbm", T * (d * eb + E * 4) + d * E * eb),
        # logits + gate in one launch (E = 128): x in, gates out, the logits stay on chip
        "replay_gate": ("hbm", T * (d * eb + K * idx_bytes + K * 4) + d * E * eb),
        "permute_index": ("hbm", T * K * (2 * idx_bytes + 8)),
        "gather_rows": ("hbm", T * (d * eb + K * d * eb + K * 4)),
        "combine": ("hbm", T * (K * d * eb + d * eb + K * 8)),
        "gate_backward": ("hbm", T * (K * (nparts * 4 + 4 + 4 + idx_bytes) + K * 4 + 2 * E * eb)),
        "dx_finish": ("hbm", T * (K * d * eb + d * eb + K * 12) + E * d * eb),
        "router_wgrad": ("mfma", 2.0 * T * d * E),
        "ffn1_swiglu": ("mfma", 4.0 * S * d * F),
        "ffn2_down": ("mfma", 2.0 * S * d * F),
        "ffn_dh": ("mfma", 2.0 * S * d * F),
        "ffn_dxp": ("mfma", 4.0 * S * d * F),
        "ffn_wgrad_down": ("mfma", 2.0 * S * d * F),
        "ffn_wgrad_gate_up": ("mfma", 4.0 * S * d * F),   # both products in one launch
    }


def gemm_bytes(sh, backward, gated=True):
    """Algorithmic HBM bytes of one launch of each expert GEMM (operands once in, results once out).
    gated: H was saved with the gate folded in (one-call forward), so the backward writes no g*H."""
    d, E, F = sh.d, sh.E, sh.F
    S = sh.T * sh.K
    W = E * d * F * 2
    return {
        "ffn1_swiglu": S * d * 2 + 2 * W + (3 if backward else 1) * S * F * 2,
        "ffn2_down": S * F * 2 + W + S * d * 2,
        "ffn_dh": S * d * 2 + W + (5 if gated else 6) * S * F * 2,   # FA, FB, H in; dA, dB (and g*H) out
        "ffn_wgrad_down": (S * d + S * F) * 2 + 2 * W,          # f32 gradient out
        "ffn_wgrad_gate_up": (S * d + 2 * S * F) * 2 + 4 * W,
        "ffn_dxp": 2 * S * F * 2 + 2 * W + S * d * 2,
    }


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(sh, tokens, tokens_1thread):
    """The oracle, as it stands, on bounded samples of the same workload (forward + backward): `tokens`
    tokens on all host cores, then `tokens_1thread` of them on one thread."""
    import numpy as np
    from oracle import sparse
    from paper_2510_11370_amd import synth
    sub = sh.with_(T=tokens)
    L = {k: (None if v is None else v.numpy()) for k, v in synth.make_layer(sub).items()}
    s = sparse.router_logits(L["x"], L["Wr"], L["bias"])
    idx = sparse.topk_mask((s + L["noise"]).astype(np.float32), sh.K)

    def timed(n):
        t0 = time.perf_counter()
        fwd = sparse.forward(L["x"][:n], L["Wr"], idx[:n], L["Wg"], L["Wu"], L["Wd"], L["bias"])
        sparse.backward(L["dy"][:n], L["x"][:n], L["Wr"], idx[:n], L["Wg"], L["Wu"], L["Wd"], fwd)
        return time.perf_counter() - t0
    cores = sparse.num_threads()
    dt = timed(tokens)
    out = {"value": tokens / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
           "sample": "%d tokens of the same layer (all %d experts' weights), forward+backward, f64, %.1f s"
                     % (tokens, sh.E, dt),
           "cpu_model": cpu_model()}
    if tokens_1thread > 0:
        sparse.set_num_threads(1)
        n1 = min(tokens_1thread, tokens)
        dt1 = timed(n1)
        sparse.set_num_threads(cores)
        out["value_1thread"] = n1 / dt1
        out["sample_1thread"] = "%d of those tokens on one thread, %.1f s" % (n1, dt1)
    return out


def measured_ceilings(torch, r3, dev):
    """What this machine sustains on the two resources the rooflines are drawn against, measured with the
    library's calibration kernels outside the timed region: a register-only bf16 MFMA loop with constant and
    with varied operand bits (the matrix rate is power-limited and depends on the data), the same loop fed with the
    expert GEMMs' mix of LDS fragment reads and global->LDS loads (no barriers, epilogues or HBM misses: what a
    perfect schedule of that mix would reach), and a plain copy."""
    def timed(fn, reps=3):
        best = None
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            work = fn()
            b.record()
            b.synchronize()
            rate = work / (a.elapsed_time(b) * 1e-3)
            best = rate if best is None else max(best, rate)
        return best
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)

    mix_src = torch.randn(1 << 19, device=dev).to(torch.bfloat16)

    def copy():
        r3.profile_copy(dst, src)
        return 2.0 * src.numel()
    out = {"mfma_bf16_constant_operands_TFLOPs": round(timed(lambda: r3.profile_mfma(20000, False, sink)) * 1e-12, 1),
           "mfma_bf16_varied_operands_TFLOPs": round(timed(lambda: r3.profile_mfma(20000, True, sink)) * 1e-12, 1),
           "gemm_instruction_mix_TFLOPs": round(timed(lambda: r3.profile_gemm_mix(20000, mix_src, sink)) * 1e-12, 1),
           "gemm_instruction_mix_4waves_128x128_TFLOPs": round(
               timed(lambda: r3.profile_gemm_mix(20000, mix_src, sink, shape=1)) * 1e-12, 1),
           "hbm_copy_GBs": round(timed(copy) * 1e-9, 1)}
    del src, dst
    return out


def bench_diagnostics(args, torch, r3, dev):
    """Secondary workload: the Section 3 diagnostics on a record pair of the 48-layer configuration's size and
    on 10 M token log-probabilities (the sample size of the paper's scatter plot)."""
    L, T, K, E, n = 48, 131072, 8, 128, 10_000_000
    g = torch.Generator(device=dev).manual_seed(1)
    a = torch.rand(L, T, E, generator=g, device=dev).argsort(dim=2)[:, :, :K].sort(dim=2).values.to(torch.uint8)
    b = a.clone()
    hit = torch.rand(L, T, generator=g, device=dev) < 0.1
    b[hit] = torch.rand(int(hit.sum()), E, generator=g, device=dev).argsort(dim=1)[:, :K].to(torch.uint8)
    D = r3.desc(T, 16, E, K, 16)
    hist = torch.zeros(K + 1, dtype=torch.int64, device=dev)
    tc = torch.empty(T, dtype=torch.int32, device=dev)
    tr = torch.empty(T, dtype=torch.int32, device=dev)
    so = torch.arange(0, T + 1, 2048, dtype=torch.int32, device=dev)
    sm = torch.empty(so.numel() - 1, dtype=torch.float64, device=dev)
    li = torch.log(torch.rand(n, generator=g, device=dev).clamp_min(1e-4))
    lt = li + 0.05 * torch.randn(n, generator=g, device=dev)
    kl = torch.zeros(1, dtype=torch.float64, device=dev)
    taus = [1.0, 1.5, 2.0, 4.0, 10.0]
    frac = torch.zeros(len(taus), dtype=torch.float64, device=dev)
    ws = torch.empty(256 << 10, dtype=torch.uint8, device=dev)

    def step():
        r3.routing_diff(D, L, a, b, T * K, hist, tc, tr, so, sm)
        r3.policy_discrepancy(lt, li, taus, kl, frac, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    r3.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = r3.profile_read()
    r3.profile_enable(False)
    work = {"routing_diff": 2 * L * T * K + 8 * T, "policy_discrepancy": 8 * n}
    kernels = {}
    for name, (ms, cnt) in prof.items():
        gbs = work[name] / (ms / cnt) * 1e-6
        kernels[name] = {"bound": "hbm", "avg_ms": round(ms / cnt, 4), "launches_per_step": cnt // args.steps,
                         "achieved": round(gbs, 1), "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4)}
    ms_per_step = wall * 1e3 / args.steps
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    print(json.dumps({
        "metric": "routers compared/sec (two 48x131072x8 records) with a 10M-token policy discrepancy, 1 GPU",
        "value": round(L * T / (ms_per_step * 1e-3), 1), "unit": "routers/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic (seeded)",
        "config": {"workload": "diagnostics: routing_diff L=48 T=131072 K=8 E=128 uint8 + policy_discrepancy n=1e7",
                   "kl_k3": kl.item(), "F_tau": dict(zip(map(str, taus), frac.cpu().tolist()))},
        "roofline": {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["achieved"], "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": kernels[dom]["frac"], "traffic": None},
        "kernels": kernels}))


def bench_mask_cache(args, torch, r3, synth, dev):
    """Secondary workload: the Section 4.2 mask cache at the 48-layer configuration's size.  One step stores the
    masks of every token the batch's sequences own (a rollout's worth, handed over layer-major as the per-layer
    recording leaves them) and gathers the packed batch's layer-major record back through the block table."""
    import numpy as np
    L, T, K, E, P = 48, 131072, 8, 128, 16
    lens, shared, table_np, num_pages = synth.rollout_batch(T, P, group=4, seed=3)
    start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seq_id = np.concatenate([np.full(int(n - sh), s, np.int32) for s, (n, sh) in enumerate(zip(lens, shared))])
    pos = np.concatenate([np.arange(sh, n, dtype=np.int32) for n, sh in zip(lens, shared)])
    n = len(seq_id)
    g = torch.Generator(device=dev).manual_seed(2)
    new = torch.randint(0, E, (L, n, K), generator=g, device=dev).to(torch.uint8)
    pages = torch.zeros((num_pages, P, L, K), dtype=torch.uint8, device=dev)
    table = torch.from_numpy(table_np).to(dev)
    d_seq, d_pos, d_start = (torch.from_numpy(a).to(dev) for a in (seq_id, pos, start))
    out = torch.empty((L, T, K), dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)

    def step():
        r3.mask_cache_append(pages, table, d_seq, d_pos, new, n * K, K, status)
        r3.mask_cache_gather(pages, table, d_start, out, status)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    r3.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = r3.profile_read()
    r3.profile_enable(False)
    assert int(status.item()) == 0
    work = {"mask_cache_append": 2 * n * L * K + 8 * n, "mask_cache_gather": 2 * T * L * K}
    kernels = {}
    for name, (ms, cnt) in prof.items():
        gbs = work[name] / (ms / cnt) * 1e-6
        kernels[name] = {"bound": "hbm", "avg_ms": round(ms / cnt, 4), "launches_per_step": cnt // args.steps,
                         "achieved": round(gbs, 1), "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4)}
    ms_per_step = wall * 1e3 / args.steps
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    print(json.dumps({
        "metric": "tokens' masks stored and gathered/sec (48 layers x top-8 uint8, paged, 1 GPU)",
        "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic (seeded)",
        "config": {"workload": "mask_cache: L=48 T=131072 K=8 uint8, page 16 tokens, %d sequences in groups of 4 "
                               "with shared prompts (%d tokens come from shared pages), %d pages"
                               % (len(lens), int(shared.sum()), num_pages)},
        "roofline": {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["achieved"], "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": kernels[dom]["frac"], "traffic": None},
        "kernels": kernels}))


def stored_traffic(workload, kernel):
    """HBM bytes per launch (fetch + write) of `kernel` from the committed counter summary of this workload
    (two rocprofv3 --pmc runs of this script, scaled by the calibration copy), or None if there is none."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "%s_hbm_traffic.md" % workload)
    try:
        for line in open(path):
            f = [c.strip() for c in line.split("|")]
            if len(f) >= 5 and f[1] == kernel:
                return {"fetch_bytes": float(f[2]), "write_bytes": float(f[3]), "bytes": float(f[4]),
                        "source": "profiles/%s_hbm_traffic.md" % workload}
    except (OSError, ValueError):
        pass
    return None


def run_layer(args, workload, torch, r3, synth, calib_copy=False):
    """Time `workload` (a key of synth.CONFIGS): W warm-up steps, then exactly K timed steps; returns the
    result block (metric line fields, per-kernel table, roofline of the dominant expert GEMM)."""
    sh = synth.CONFIGS[workload]
    dev = "cuda"
    bwd = not args.forward_only and workload in ("fwdbwd_16k", "zipf_64k")
    L = sh.layers
    D = r3.desc(sh.T, sh.d, sh.E, sh.K, sh.F, sh.act)
    adt = r3.act_dtype(D)
    t = {k: synth.draw(sh, k, dev).to(adt) for k in ("x", "Wg", "Wu", "Wd")}
    Wr = [synth.draw(sh, "Wr", dev, layer=l).to(adt) for l in range(L)]
    dy = synth.draw(sh, "dy", dev).to(adt) if bwd else None
    bias = synth.draw(sh, "bias", dev)
    buf = r3.LayerBuffers(D, backward=bwd, gathered_copy=args.gathered_copy)   # default: rows gathered inside the GEMMs
    record = torch.zeros(L, sh.T, sh.K, dtype=r3.idx_torch_dtype(D), device=dev)   # layer-major record
    agree = torch.zeros(L, 2, dtype=torch.int64, device=dev)

    def next_x(x, y):
        """Harness glue between stacked layers: residual, then unit RMS per token (stands in for the rest
        of a transformer block; the expert FFN is quadratic in its input, a bare residual chain overflows)."""
        if adt == torch.bfloat16:   # two passes over the activations instead of eight: this is glue, not the method
            return torch.nn.functional.rms_norm(x + y, (x.shape[1],), None, 1e-6)
        r = x.float() + y.float()
        return (r * torch.rsqrt(r.pow(2).mean(dim=1, keepdim=True) + 1e-6)).to(adt)

    # the rollout engine's view, made once: inference logits = training logits + noise, per layer
    s_infer = []
    logits = torch.empty(sh.T, sh.E, dtype=torch.float32, device=dev)
    x = t["x"]
    for l in range(L):
        r3.replay_gate(D, x, Wr[l], record[l], buf.gates, bias=bias, logits_out=logits, ws=buf.ws_gate)
        s_infer.append(logits + synth.draw(sh, "noise", dev, layer=l))
        if L > 1:
            r3.record_topk(D, s_infer[l], record[l], buf.status)
            x = next_x(x, r3.forward(buf, x, Wr[l], record[l], t["Wg"], t["Wu"], t["Wd"], bias=bias))
    del logits
    buf.status.zero_()      # (the first gate calls above ran on a record that was not made yet)

    # the forward: one C call (r3_moe_forward, gate folded into the expert network) unless --six-calls
    fwd_call = r3.forward if (args.six_calls or args.gathered_copy) else r3.forward_one_call

    def step():
        x = t["x"]
        for l in range(L):
            r3.record_topk(D, s_infer[l], record[l], buf.status)
            y = fwd_call(buf, x, Wr[l], record[l], t["Wg"], t["Wu"], t["Wd"], bias=bias,
                         agree_out=agree[l] if L > 1 else None)
            if bwd:
                r3.backward(buf, dy, x, Wr[l], record[l], t["Wg"], t["Wu"], t["Wd"])
            if L > 1:
                x = next_x(x, y)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        # the step captured once in a HIP graph and replayed: the timed region is --steps replays; the per-kernel
        # events come from a second, eager pass of the same length that is not part of `value`
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        r3.profile_enable(True)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
    else:
        # timed region: exactly --steps steps, per-kernel HIP events recorded inside the library
        r3.profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    prof = r3.profile_read()
    r3.profile_enable(False)
    assert int(buf.status.item()) == 0, "device status word set"
    if calib_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        r3.profile_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    counts = buf.counts.cpu()

    ms_per_step = wall * 1e3 / args.steps
    work = kernel_work(sh, 1 if D.idx == r3.IDX_U8 else 2)
    gbytes = gemm_bytes(sh, bwd, gated=fwd_call is r3.forward_one_call)
    kernels = {}
    for name, (ms, n) in prof.items():
        kind, amount = work[name]
        avg_ms = ms / n
        if kind == "mfma":
            ach, peak, unit = amount / avg_ms * 1e-9, PEAK_BF16_TFLOPS, "TFLOP/s"
        else:
            ach, peak, unit = amount / avg_ms * 1e-6, PEAK_HBM_GBS, "GB/s"
        kernels[name] = {"bound": kind, "avg_ms": round(avg_ms, 4), "launches_per_step": n // args.steps,
                         "achieved": round(ach, 1), "unit": unit, "frac": round(ach / peak, 4)}
        if name in gbytes:   # the expert GEMMs sit near the ridge: their share of HBM peak as well
            kernels[name]["hbm_GBps"] = round(gbytes[name] / avg_ms * 1e-6, 1)
            kernels[name]["hbm_frac"] = round(gbytes[name] / avg_ms * 1e-6 / PEAK_HBM_GBS, 4)
    mfma = {k: v for k, v in kernels.items() if v["bound"] == "mfma" and k.startswith("ffn")}
    dom = max(mfma, key=lambda k: mfma[k]["avg_ms"] * mfma[k]["launches_per_step"]) if mfma else None
    roofline = None
    if dom:
        kd = kernels[dom]
        roofline = {"kernel": dom, "bound": "mfma", "achieved": kd["achieved"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": kd["frac"], "traffic": None}
        tr = stored_traffic(workload, dom)
        if tr:   # HBM bytes per launch (fetch + write) from the committed counter summary
            roofline.update(traffic=tr["bytes"], traffic_fetch_bytes=tr["fetch_bytes"],
                            traffic_write_bytes=tr["write_bytes"], traffic_source=tr["source"],
                            algorithmic_hbm_bytes=gbytes.get(dom))
        # every expert GEMM of the step together: algorithmic FLOP over the sum of their times
        tot_ms = sum(v["avg_ms"] * v["launches_per_step"] for v in mfma.values())
        tot_fl = sum(work[k][1] * v["launches_per_step"] for k, v in mfma.items())
        roofline["all_expert_gemms_TFLOPs"] = round(tot_fl / tot_ms * 1e-9, 1)
        roofline["all_expert_gemms_frac"] = round(tot_fl / tot_ms * 1e-9 / PEAK_BF16_TFLOPS, 4)
    out = {
        "metric": "tokens/sec for R3 replayed MoE layer fwd+bwd at 1 GPU",
        "value": round(sh.T * L / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": sh.act,
        "data": "synthetic (seeded; shape of a 128-expert top-8 MoE layer)",
        "config": {"workload": "%s: T=%d d=%d E=%d K=%d F=%d %s%s, record+forward%s" % (
            workload, sh.T, sh.d, sh.E, sh.K, sh.F, sh.act, " x %d layers" % L if L > 1 else "",
            "+backward" if bwd else "") + (", Zipf(%.1f) router bias" % sh.zipf_s if sh.zipf_s else "")
            + (", launched as a HIP graph" if args.graph else ""),
            "rows_per_expert_min_mean_max": [int(counts.min()), float(counts.float().mean()), int(counts.max())]},
        "roofline": roofline, "kernels": kernels,
    }
    if L > 1:   # value counts token-layers per second; agreement = tokens whose own top-K is the replayed set
        agree.zero_()
        step()
        rate = (agree[:, 0].double() / sh.T).cpu()
        out["config"]["agreement_rate_per_layer_min_mean_max"] = [round(float(rate.min()), 4),
                                                                  round(float(rate.mean()), 4),
                                                                  round(float(rate.max()), 4)]
        out["metric"] = "token-layers/sec for R3 record+replay forward over a %d-layer stack at 1 GPU" % L
    del buf, t, Wr, dy, record, s_infer
    torch.cuda.empty_cache()
    return out


DEFAULT_WORKLOAD = "zipf_64k"      # the largest forward+backward configuration
ALSO_WORKLOAD = "fwdbwd_16k"       # timed in the same run when no --workload is given


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    help="one of the configurations (fwd_4k, fwdbwd_16k, stack48_128k, zipf_64k), diagnostics or "
                         "mask_cache; default: zipf_64k, with fwdbwd_16k timed alongside")
    ap.add_argument("--cpu-tokens", type=int, default=4096, help="tokens of the oracle's timed sample (0 = skip)")
    ap.add_argument("--cpu-tokens-1thread", type=int, default=256,
                    help="tokens of that sample timed again on one thread (0 = skip)")
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--gathered-copy", action="store_true",
                    help="materialise the expert-sorted copy of the tokens (Xp) instead of reading x through the "
                         "permutation inside the expert GEMMs")
    ap.add_argument("--six-calls", action="store_true",
                    help="run the forward as r3_replay_gate, r3_permute, r3_grouped_ffn, r3_combine instead of the "
                         "one-call r3_moe_forward (the backward then also scales H by the gates itself)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of the step captured in a HIP graph (single-layer workloads) instead of "
                         "eager launches")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the calibration kernels after the timed region")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region, run one plain 256 MiB copy kernel (reference point for "
                         "hardware traffic counters collected around this command)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_2510_11370_amd import r3, synth
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if args.workload == "diagnostics":
        return bench_diagnostics(args, torch, r3, "cuda")
    if args.workload == "mask_cache":
        return bench_mask_cache(args, torch, r3, synth, "cuda")
    workload = args.workload or DEFAULT_WORKLOAD
    out = run_layer(args, workload, torch, r3, synth, calib_copy=args.calib_copy)
    if args.workload is None:
        time.sleep(3.0)   # let the card's power and clock state settle after the first workload
        also = run_layer(args, ALSO_WORKLOAD, torch, r3, synth)
        out["config"]["workload"] += ("  [the line's value; the block under also.%s is the 16384-token "
                                      "forward+backward configuration, same run, same steps and warm-up]" % ALSO_WORKLOAD)
        out["also"] = {ALSO_WORKLOAD: {k: also[k] for k in ("value", "unit", "ms_per_step", "config", "roofline",
                                                             "kernels")}}
    roofline = out["roofline"]
    if not args.no_ceilings:
        out["ceilings"] = measured_ceilings(torch, r3, "cuda")
        for rf in [roofline] + [b["roofline"] for b in out.get("also", {}).values()]:
            if rf:   # context only: the same achieved rate against what this machine sustains on such data
                rf["frac_of_measured_ceiling"] = round(
                    rf["achieved"] / out["ceilings"]["mfma_bf16_varied_operands_TFLOPs"], 4)
                rf["frac_of_instruction_mix_ceiling"] = round(
                    rf["achieved"] / out["ceilings"]["gemm_instruction_mix_TFLOPs"], 4)
    if args.cpu_tokens > 0:
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(synth.CONFIGS[workload], args.cpu_tokens, args.cpu_tokens_1thread)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
