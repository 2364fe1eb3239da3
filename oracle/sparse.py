"""ctypes wrapper over r3_oracle.c (test infrastructure; see the C file's header).

Arrays are NumPy: float32 for the layer's inputs (bf16-rounded values are exact
in float32), int32 for expert ids and permutations, float64 for every result.
"""
import ctypes as C

import numpy as np

from .build import build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads():
    return int(lib().oracle_num_threads())


def set_num_threads(n):
    lib().oracle_set_num_threads(C.c_int(int(n)))


def router_logits(x, Wr, bias=None):
    """s = x Wr (+ bias): Section 4.1, router-logit equation."""
    x, Wr = _f32(x), _f32(Wr)
    T, d = x.shape
    E = Wr.shape[1]
    assert Wr.shape[0] == d
    bias = None if bias is None else _f32(bias)
    s = np.empty((T, E), np.float64)
    lib().oracle_router_logits(T, d, E, _p(x), _p(Wr), _p(bias), _p(s))
    return s


def topk_mask(logits, K):
    """TopKMask(s, K) as K ascending expert ids per token."""
    T, E = logits.shape
    idx = np.empty((T, K), np.int32)
    if logits.dtype == np.float32:
        lg = _f32(logits)
        lib().oracle_topk_mask_f32(T, E, K, _p(lg), _p(idx))
    else:
        lg = _f64(logits)
        lib().oracle_topk_mask_f64(T, E, K, _p(lg), _p(idx))
    return idx


def replay_gate(s, idx):
    """Replay gate: softmax of the training logits over the recorded set."""
    s, idx = _f64(s), _i32(idx)
    T, E = s.shape
    K = idx.shape[1]
    assert idx.min() >= 0 and idx.max() < E
    g = np.empty((T, K), np.float64)
    lib().oracle_replay_gate(T, E, K, _p(s), _p(idx), _p(g))
    return g


def permute(idx, E):
    idx = _i32(idx)
    T, K = idx.shape
    assert idx.min() >= 0 and idx.max() < E
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    inv_perm = np.empty(T * K, np.int32)
    perm = np.empty(T * K, np.int32)
    lib().oracle_permute(T, E, K, _p(idx), _p(counts), _p(offsets), _p(inv_perm), _p(perm))
    return counts, offsets, inv_perm, perm


def gather_rows(x, perm, K):
    x, perm = _f32(x), _i32(perm)
    T, d = x.shape
    Xp = np.empty((T * K, d), np.float32)
    lib().oracle_gather_rows(T, K, d, _p(x), _p(perm), _p(Xp))
    return Xp


def grouped_ffn(Xp, offsets, Wg, Wu, Wd):
    """Per-expert SwiGLU on the expert's row segment; returns a, b, h, o."""
    Xp, offsets = _f32(Xp), _i32(offsets)
    Wg, Wu, Wd = _f32(Wg), _f32(Wu), _f32(Wd)
    E, d, F = Wg.shape
    assert Wu.shape == (E, d, F) and Wd.shape == (E, F, d) and Xp.shape[1] == d
    S = Xp.shape[0]
    assert offsets[0] == 0 and offsets[-1] == S
    a = np.zeros((S, F), np.float64)
    b = np.zeros((S, F), np.float64)
    h = np.zeros((S, F), np.float64)
    o = np.zeros((S, d), np.float64)
    lib().oracle_grouped_ffn(E, d, F, _p(offsets), _p(Xp), _p(Wg), _p(Wu), _p(Wd),
                             _p(a), _p(b), _p(h), _p(o))
    return a, b, h, o


def combine(o, g, inv_perm):
    o, g, inv_perm = _f64(o), _f64(g), _i32(inv_perm)
    T, K = g.shape
    d = o.shape[1]
    y = np.empty((T, d), np.float64)
    lib().oracle_combine(T, K, d, _p(o), _p(g), _p(inv_perm), _p(y))
    return y


def forward(x, Wr, idx, Wg, Wu, Wd, bias=None):
    """The whole replayed forward; returns a dict with every intermediate."""
    x, Wr, idx = _f32(x), _f32(Wr), _i32(idx)
    Wg, Wu, Wd = _f32(Wg), _f32(Wu), _f32(Wd)
    bias = None if bias is None else _f32(bias)
    T, d = x.shape
    E, _, F = Wg.shape
    K = idx.shape[1]
    assert idx.min() >= 0 and idx.max() < E
    S = T * K
    r = dict(
        s=np.empty((T, E), np.float64), g=np.empty((T, K), np.float64),
        counts=np.empty(E, np.int32), offsets=np.empty(E + 1, np.int32),
        inv_perm=np.empty(S, np.int32), perm=np.empty(S, np.int32),
        Xp=np.empty((S, d), np.float32), a=np.zeros((S, F), np.float64),
        b=np.zeros((S, F), np.float64), h=np.zeros((S, F), np.float64),
        o=np.zeros((S, d), np.float64), y=np.empty((T, d), np.float64))
    lib().oracle_moe_forward(T, d, E, K, F, _p(x), _p(Wr), _p(bias), _p(idx), _p(Wg),
                             _p(Wu), _p(Wd), _p(r["s"]), _p(r["g"]), _p(r["counts"]),
                             _p(r["offsets"]), _p(r["inv_perm"]), _p(r["perm"]),
                             _p(r["Xp"]), _p(r["a"]), _p(r["b"]), _p(r["h"]), _p(r["o"]),
                             _p(r["y"]))
    return r


def backward(dy, x, Wr, idx, Wg, Wu, Wd, fwd, want_dbias=False):
    """Gradients of sum(dy*y) w.r.t. x and every weight, recorded mask constant."""
    dy, x, Wr, idx = _f32(dy), _f32(x), _f32(Wr), _i32(idx)
    Wg, Wu, Wd = _f32(Wg), _f32(Wu), _f32(Wd)
    T, d = x.shape
    E, _, F = Wg.shape
    K = idx.shape[1]
    S = T * K
    r = dict(
        dO=np.zeros((S, d), np.float64), dz=np.empty((T, K), np.float64),
        ds=np.empty((T, E), np.float64), dxr=np.empty((T, d), np.float64),
        da=np.zeros((S, F), np.float64), db=np.zeros((S, F), np.float64),
        dXp=np.zeros((S, d), np.float64), dx=np.empty((T, d), np.float64),
        dWr=np.empty((d, E), np.float64),
        dbias=np.empty(E, np.float64) if want_dbias else None,
        dWg=np.zeros((E, d, F), np.float64), dWu=np.zeros((E, d, F), np.float64),
        dWd=np.zeros((E, F, d), np.float64))
    lib().oracle_moe_backward(
        T, d, E, K, F, _p(dy), _p(x), _p(Wr), _p(idx), _p(Wg), _p(Wu), _p(Wd),
        _p(_f64(fwd["g"])), _p(_i32(fwd["offsets"])), _p(_i32(fwd["inv_perm"])),
        _p(_f32(fwd["Xp"])), _p(_f64(fwd["a"])), _p(_f64(fwd["b"])), _p(_f64(fwd["h"])),
        _p(_f64(fwd["o"])), _p(r["dO"]), _p(r["dz"]), _p(r["ds"]), _p(r["dxr"]),
        _p(r["da"]), _p(r["db"]), _p(r["dXp"]), _p(r["dx"]), _p(r["dWr"]),
        _p(r["dbias"]), _p(r["dWg"]), _p(r["dWu"]), _p(r["dWd"]))
    return r


def agreement(idx_a, idx_b):
    """(tokens with equal expert sets, total shared experts) of two records."""
    idx_a, idx_b = _i32(idx_a), _i32(idx_b)
    T, K = idx_a.shape
    out = np.zeros(2, np.int64)
    lib().oracle_agreement(T, K, _p(idx_a), _p(idx_b), _p(out))
    return int(out[0]), int(out[1])


def gate_backward(dy, o, g, idx, inv_perm, E):
    """Backward through combine and masked softmax: returns dO, dz, ds."""
    dy, o, g, idx, inv_perm = _f32(dy), _f64(o), _f64(g), _i32(idx), _i32(inv_perm)
    T, d = dy.shape
    K = idx.shape[1]
    dO = np.zeros((T * K, d), np.float64)
    dz = np.empty((T, K), np.float64)
    ds = np.empty((T, E), np.float64)
    lib().oracle_gate_backward(T, d, E, K, _p(dy), _p(o), _p(g), _p(idx), _p(inv_perm), _p(dO), _p(dz),
                               _p(ds))
    return dO, dz, ds


def grouped_ffn_backward(Xp, offsets, Wg, Wu, Wd, a, b, h, dO):
    """Expert backward on row segments: returns da, db, dXp, dWg, dWu, dWd."""
    Xp, offsets = _f32(Xp), _i32(offsets)
    Wg, Wu, Wd = _f32(Wg), _f32(Wu), _f32(Wd)
    E, d, F = Wg.shape
    S = Xp.shape[0]
    da = np.zeros((S, F), np.float64)
    db = np.zeros((S, F), np.float64)
    dXp = np.zeros((S, d), np.float64)
    dWg = np.zeros((E, d, F), np.float64)
    dWu = np.zeros((E, d, F), np.float64)
    dWd = np.zeros((E, F, d), np.float64)
    lib().oracle_grouped_ffn_backward(E, d, F, _p(offsets), _p(Xp), _p(Wg), _p(Wu), _p(Wd), _p(_f64(a)),
                                      _p(_f64(b)), _p(_f64(h)), _p(_f64(dO)), _p(da), _p(db), _p(dXp),
                                      _p(dWg), _p(dWu), _p(dWd))
    return da, db, dXp, dWg, dWu, dWd
