"""Shared helpers of the parity tests: build a seeded case on both sides, compare."""
import os

import numpy as np
import torch

from oracle import sparse
from paper_2510_11370_amd import r3, synth

# Floating-point bars of this build: bf16 tensors rel err <= 1e-2, f32 gates <= 1e-5.
# f32 activations (config 1) are held to 2e-4: f32 accumulation against the f64 oracle.
REL = {"bf16": 1e-2, "f32": 2e-4}


# Element bar: |gpu-ref| <= rel |ref| + ELEM_C rel s_ij, where s_ij = rms(row i) rms(column j) / rms(ref) is
# the magnitude an element at (i, j) has when rows and columns each carry their own scale.  The second
# term is the room for the rounding noise of the bf16 tensors a result passes through (H, Yp, dA/dB, ...
# each carry up to 2^-9 of their value; summed over a contraction that is a few 1e-3 of the output's local
# magnitude, normally distributed).  A tensor-wide rms is the wrong yardstick: SwiGLU rows (tokens) are
# heavy-tailed, the columns of dW_r (experts) differ by their load, and the weight gradient of an expert
# with a handful of rows is a sum of as few outer products, large where both factors are.  ELEM_C = 1 is
# about 3.5 sigma of the measured noise (normwise error 2.9e-3 for the weight gradients): tensors of
# 1e6..1e8 elements then fail on a few hundred elements by chance.  Measured over the full-size cases
# (about 1e9 compared elements; R3_TOL_LOG records what each call needs): the weight gradients need up to
# 2.0 on a single element in 6e8, every other tensor less.
ELEM_C = 2.5


def _log(line):
    path = os.environ.get("R3_TOL_LOG")
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def assert_close(gpu, ref, name, rel, sigma=None, elem_c=None):
    """The floating-point bar for tensors in the activation dtype and for weight gradients.

    1. whole tensor, norm-wise:  |gpu-ref|_2 <= rel |ref|_2                (the stated bar)
    2. every row (last dim), norm-wise: <= 2 rel |row|_2 + rel rms(ref) sqrt(n)
       (a single wrong token or feature row cannot hide in the tensor norm)
    3. every element: |gpu-ref| <= rel |ref| + ELEM_C rel rms(row) rms(column) / rms(ref)
       (a misplaced element is off by about the magnitude its row and column have; with fewer than 16
       rows the column factor is dropped: rms(row) alone)
    `sigma` (same shape as ref, optional): modelled standard deviation of the error that the bf16
    storage of an upstream tensor induces in this one; 8 sigma is added to bars 2 and 3.  Used for the
    router gradients, where a token's dz = g (dg - sum g dg) is a difference of nearly equal numbers
    and an expert chosen by one or two tokens has no other terms to average that error away.
    With R3_TOL_LOG=<file> every call appends how much of each bar it used.
    """
    c = ELEM_C if elem_c is None else elem_c
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (name, gpu.shape, ref.shape)
    assert np.isfinite(gpu).all(), name
    n = ref.shape[-1] if ref.ndim >= 1 else 1
    diff = np.abs(gpu - ref).reshape(-1, n)
    ref2 = ref.reshape(-1, n)
    nref = np.linalg.norm(ref2)
    err = np.linalg.norm(diff)
    rms = max(nref / np.sqrt(max(ref.size, 1)), 1e-300)
    rerr = np.linalg.norm(diff, axis=1)
    rref = np.linalg.norm(ref2, axis=1)
    sig = None if sigma is None else np.asarray(sigma, np.float64).reshape(-1, n)
    rslack = 0.0 if sig is None else 8 * np.linalg.norm(sig, axis=1)
    row_use = rerr / np.maximum(2 * rel * rref + rel * rms * np.sqrt(n) + rslack, 1e-300)
    # element bar: what multiple of rel * s_ij each element needs beyond rel*|ref| (and the sigma term)
    rrms = rref / np.sqrt(n)
    # (a column's magnitude cannot be told from a handful of rows: below 16 rows the row scale alone is used)
    crms = np.linalg.norm(ref2, axis=0) / np.sqrt(ref2.shape[0]) if ref2.shape[0] >= 16 else np.full(n, rms)
    scale = np.maximum(rrms[:, None] * crms[None, :] / rms, 1e-300)
    over = diff - rel * np.abs(ref2)
    need_plain = (over / (rel * scale)).max() if over.size else 0.0
    n_sigma = 0
    if sig is not None:
        n_sigma = int((over > c * rel * scale).sum())          # elements that lean on the sigma term
        over = over - 8 * sig
    need = (over / (rel * scale)).max() if over.size else 0.0
    _log("%-34s n=%-10d normwise %.2e (bar %.0e)  worst row %.2f of bar 2  element bar needs c=%.2f%s" % (
        name, ref.size, err / max(nref, 1e-300), rel, row_use.max() if row_use.size else 0.0, need,
        "" if sig is None else " (c=%.2f without the 8-sigma term; %d elements lean on it)" % (need_plain, n_sigma)))
    assert err <= rel * nref + 1e-30, "%s: normwise rel err %.3e > %.1e" % (name, err / max(nref, 1e-300), rel)
    if ref.ndim >= 2:
        assert not (row_use > 1).any(), "%s: %d rows outside tolerance (worst row rel err %.3e)" % (
            name, (row_use > 1).sum(), (rerr / np.maximum(rref, 1e-300)).max())
    bad = over > c * rel * scale
    assert not bad.any(), "%s: %d of %d elements outside tolerance (max abs err %.3e, rms %.3e, needs c=%.2f)" % (
        name, bad.sum(), bad.size, diff.max(), rms, need)
    return err / max(nref, 1e-300)


def router_gradient_sigma(x, dy, idx, fwd, E):
    """Error model for dW_r and dbias under bf16 storage of the expert activations: each element of o
    carries its own rounding error (uniform within half an ulp: relative std 2^-9 / sqrt(3)) and, through
    the down projection, that of the bf16-stored H, which for random-sign sums is as large again:
      var(dg_j) = 2 u^2 sum_c dy_c^2 o_jc^2,   dz_j = g_j (dg_j - sum_i g_i dg_i)  =>
      var(dz_j) = g_j^2 ((1 - g_j)^2 var(dg_j) + sum_{i != j} g_i^2 var(dg_i)),
    scattered to the dense ds and pushed through dW_r = x^T ds, dbias = sum_t ds.
    Returns (sigma of dW_r [d,E], sigma of dbias [E]).  Oracle quantities only."""
    x, dy = np.asarray(x, np.float64), np.asarray(dy, np.float64)
    T, K = idx.shape
    u2 = 2.0 * (2.0 ** -9) ** 2 / 3.0
    o = np.asarray(fwd["o"], np.float64)[np.asarray(fwd["inv_perm"]).reshape(T, K)]      # [T,K,d]
    g = np.asarray(fwd["g"], np.float64)
    vdg = u2 * np.einsum("tc,tkc->tk", dy * dy, o * o)
    tot = (g * g * vdg).sum(axis=1, keepdims=True)
    vdz = g * g * ((1 - g) ** 2 * vdg + tot - g * g * vdg)
    vds = np.zeros((T, E))
    np.put_along_axis(vds, idx.astype(np.int64), vdz, axis=1)
    return np.sqrt((x * x).T @ vds), np.sqrt(vds.sum(axis=0))


def assert_gates_close(gpu, ref):
    """|g - g_ref| <= 1e-5 g_ref + 1e-7 (f32 gates)."""
    gpu = np.asarray(gpu, np.float64)
    bad = np.abs(gpu - ref) > 1e-5 * ref + 1e-7
    assert not bad.any(), "gates: %d outside 1e-5 (max rel %.3e)" % (bad.sum(), (np.abs(gpu - ref) / ref).max())


def dev(a, dtype, device="cuda"):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype)


def idx_dev(idx, D, device="cuda"):
    """Expert ids as the record's compact dtype (uint8 / uint16) on the device."""
    npdt = np.uint8 if D.idx == r3.IDX_U8 else np.uint16
    return torch.from_numpy(np.ascontiguousarray(idx.astype(npdt))).to(device)


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


class Case:
    """One seeded layer: numpy float32 inputs for the oracle, device tensors for the library.

    The record is made the way the paper's rollout does: TopKMask of the inference
    logits, which here are the oracle's training logits plus seeded noise.
    """

    def __init__(self, shape, backward=True, idx_dtype=None, scale_w=1.0, device="cuda"):
        self.shape = shape
        L = synth.make_layer(shape, backward=backward)
        self.np = {k: (None if v is None else v.numpy()) for k, v in L.items()}
        if scale_w != 1.0:
            for k in ("Wg", "Wu", "Wd"):
                t = torch.from_numpy(self.np[k] * scale_w)
                self.np[k] = synth._round(t, shape.act).numpy()
        n = self.np
        self.s = sparse.router_logits(n["x"], n["Wr"], n["bias"])          # oracle training logits
        self.s_infer = (self.s + n["noise"]).astype(np.float32)             # what the rollout saw
        self.idx = sparse.topk_mask(self.s_infer, shape.K)                   # the record (oracle)
        self.D = r3.desc(shape.T, shape.d, shape.E, shape.K, shape.F, shape.act, idx_dtype)
        adt = r3.act_dtype(self.D)
        self.t = {k: dev(n[k], adt, device) for k in ("x", "Wr", "Wg", "Wu", "Wd")}
        self.t["dy"] = dev(n["dy"], adt, device) if backward else None
        self.t["bias"] = None if n["bias"] is None else dev(n["bias"], torch.float32, device)
        self.t["idx"] = idx_dev(self.idx, self.D, device)
        self.rel = REL[shape.act]
