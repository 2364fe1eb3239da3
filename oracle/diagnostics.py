"""CPU oracle of the discrepancy diagnostics (arxiv 2510.11370, Section 3) -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module; it shares
no code with the HIP path.  Plain definitions in float64 / Python sets, written for checking by eye.

* Section 3.1, "KL Divergence Estimation": the k3 estimate of KL(pi_train || pi_infer) over the response
  tokens, mean of r - 1 - log r with r = pi_train(t) / pi_infer(t).
* Section 3.1, "Extreme Token Distribution Analysis": F(tau), the share of tokens whose probability ratio
  in either direction exceeds tau.
* Section 3.2: routing differences between two records of the same tokens at router level (per token and
  layer, the number of differing expert choices), token level (per token, over all layers) and sequence
  level (per sequence, the mean over its tokens of the number of routers that differ).
"""
import numpy as np


def k3_kl(logp_train, logp_infer):
    """mean over tokens of r - 1 - log r,  r = exp(logp_train - logp_infer); inputs are float32 log-probs."""
    d = np.asarray(logp_train, np.float32).astype(np.float64) - np.asarray(logp_infer, np.float32).astype(np.float64)
    return float(np.mean(np.exp(d) - 1.0 - d)) if d.size else 0.0


def extreme_fraction(logp_train, logp_infer, taus):
    """F(tau) for each tau: share of tokens with max(r, 1/r) > tau, r = pi_train(t) / pi_infer(t).

    max(r, 1/r) > tau  <=>  |log r| > log tau, evaluated in float64: log r is the exact difference of the
    two float32 log-probabilities (exact in float64 unless their exponents are far apart), log tau the
    float64 logarithm."""
    d = np.abs(np.asarray(logp_train, np.float32).astype(np.float64) - np.asarray(logp_infer, np.float32).astype(np.float64))
    return [float(np.count_nonzero(d > np.log(np.float64(tau)))) / max(d.size, 1) for tau in taus]


def differing_choices(a, b):
    """K - |A n B| for two id lists of one router (sets of K distinct expert ids)."""
    return len(a) - len(set(int(v) for v in a) & set(int(v) for v in b))


def routing_diff(idx_a, idx_b, seq_offsets=None):
    """idx_a, idx_b: [L, T, K] expert ids of two records of the same tokens.

    Returns (router_hist [K+1]: number of (layer, token) routers with d differing choices,
             token_choices [T]: differing choices of a token summed over layers,
             token_routers [T]: number of layers in which the token's two sets differ,
             seq_mean [nseq]: mean of token_routers over the tokens of each sequence, or None)."""
    idx_a, idx_b = np.asarray(idx_a), np.asarray(idx_b)
    L, T, K = idx_a.shape
    hist = np.zeros(K + 1, np.int64)
    token_choices = np.zeros(T, np.int32)
    token_routers = np.zeros(T, np.int32)
    for l in range(L):
        for t in range(T):
            d = differing_choices(idx_a[l, t], idx_b[l, t])
            hist[d] += 1
            token_choices[t] += d
            token_routers[t] += d > 0
    seq_mean = None
    if seq_offsets is not None:
        seq_offsets = np.asarray(seq_offsets)
        seq_mean = np.zeros(len(seq_offsets) - 1, np.float64)
        for s in range(len(seq_offsets) - 1):
            lo, hi = int(seq_offsets[s]), int(seq_offsets[s + 1])
            seq_mean[s] = token_routers[lo:hi].sum() / (hi - lo) if hi > lo else 0.0
    return hist, token_choices, token_routers, seq_mean


def routing_diff_fast(idx_a, idx_b, E, seq_offsets=None):
    """The same by membership matrices (for sizes the double loop cannot finish in seconds); checked
    against routing_diff() on small inputs."""
    idx_a, idx_b = np.asarray(idx_a).astype(np.int64), np.asarray(idx_b).astype(np.int64)
    L, T, K = idx_a.shape
    token_choices = np.zeros(T, np.int64)
    token_routers = np.zeros(T, np.int64)
    hist = np.zeros(K + 1, np.int64)
    rows = np.arange(T)[:, None]
    for l in range(L):
        ma = np.zeros((T, E), bool)
        mb = np.zeros((T, E), bool)
        ma[rows, idx_a[l]] = True
        mb[rows, idx_b[l]] = True
        d = K - (ma & mb).sum(axis=1)
        hist += np.bincount(d, minlength=K + 1)
        token_choices += d
        token_routers += d > 0
    seq_mean = None
    if seq_offsets is not None:
        seq_offsets = np.asarray(seq_offsets)
        cs = np.concatenate([[0], np.cumsum(token_routers)])
        n = np.diff(seq_offsets)
        seq_mean = np.where(n > 0, (cs[seq_offsets[1:]] - cs[seq_offsets[:-1]]) / np.maximum(n, 1), 0.0)
    return hist, token_choices.astype(np.int32), token_routers.astype(np.int32), seq_mean
