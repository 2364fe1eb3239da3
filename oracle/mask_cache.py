"""CPU oracle of the router-mask cache (arxiv 2510.11370, Section 4.2) -- TEST INFRASTRUCTURE.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module; it shares
no code with the HIP path.

The paper stores, for each layer and token prefix, the routing masks next to the KV cache, so that a prefix
that hits the cache brings its masks along and nothing is re-prefilled.  Taken here as: masks live in
fixed-size pages of `P` tokens, token-major inside a page (one generated token appends its L*K ids in one
piece), addressed through the same kind of block table a paged KV cache uses (sequence -> page ids).  A
prefix shared by two sequences is the same page ids in both tables.  The training side wants one layer-major
record [L][T][K] for a packed batch of sequences.

Plain Python loops, written for checking by eye.
"""
import numpy as np


def append(pages, P, block_table, seq_id, position, idx_new):
    """Write the ids of n new tokens: token i of sequence seq_id[i] at position[i] (0-based in its sequence)
    goes to page block_table[seq_id[i]][position[i] // P], slot position[i] % P.
    pages: [num_pages, P, L, K] (modified in place); idx_new: [n, L, K]."""
    for i in range(len(seq_id)):
        page = int(block_table[seq_id[i]][position[i] // P])
        assert page >= 0
        pages[page, position[i] % P] = idx_new[i]
    return pages


def gather(pages, P, block_table, seq_start):
    """Layer-major record [L, T, K] of a packed batch: sequence s owns tokens seq_start[s]..seq_start[s+1]
    and token j of it is read from page block_table[s][j // P], slot j % P."""
    _, _, L, K = pages.shape
    T = int(seq_start[-1])
    out = np.zeros((L, T, K), pages.dtype)
    for s in range(len(seq_start) - 1):
        for j in range(int(seq_start[s + 1]) - int(seq_start[s])):
            page = int(block_table[s][j // P])
            assert page >= 0
            out[:, int(seq_start[s]) + j, :] = pages[page, j % P]
    return out
