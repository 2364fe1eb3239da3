"""Dense brute force of the replayed MoE layer in NumPy float64 (test infrastructure).

The equations of arxiv 2510.11370, Section 4.1, written with dense E-vectors:
every expert runs on every token and the recorded routing enters only as a 0/1
mask.  No permutation, no grouping, no sparsity.  Use on tiny shapes only.
"""
import numpy as np


def mask_from_idx(idx, E):
    """Dense 0/1 mask I in {0,1}^E per token from the K recorded expert ids."""
    T, K = idx.shape
    m = np.zeros((T, E), np.float64)
    for t in range(T):
        for j in range(K):
            m[t, idx[t, j]] = 1.0
    return m


def replay_gate_dense(s, mask):
    """g_i = I_i exp(s_i) / sum_j I_j exp(s_j), written exactly so (no max shift)."""
    w = mask * np.exp(s)
    return w / w.sum(axis=1, keepdims=True)


def expert(xv, Wg, Wu, Wd):
    """SwiGLU expert on a batch of rows: W_down(silu(x W_gate) * (x W_up))."""
    a = xv @ Wg
    b = xv @ Wu
    return ((a / (1.0 + np.exp(-a))) * b) @ Wd


def forward(x, Wr, idx, Wg, Wu, Wd, bias=None):
    """y = sum_{i=1..E} g_replay,i * E_i(x), all E experts evaluated."""
    x = np.asarray(x, np.float64)
    Wr = np.asarray(Wr, np.float64)
    E = Wg.shape[0]
    s = x @ Wr
    if bias is not None:
        s = s + np.asarray(bias, np.float64)
    g = replay_gate_dense(s, mask_from_idx(np.asarray(idx), E))
    y = np.zeros_like(x)
    for i in range(E):
        y += g[:, i:i + 1] * expert(x, np.asarray(Wg[i], np.float64),
                                    np.asarray(Wu[i], np.float64),
                                    np.asarray(Wd[i], np.float64))
    return s, g, y
