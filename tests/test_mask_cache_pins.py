"""Pins of the mask-cache oracle (oracle/mask_cache.py): round trips, prefix sharing, page boundaries."""
import numpy as np

from oracle import mask_cache as mc


def _ids(n, L, K, E, seed):
    rng = np.random.default_rng(seed)
    return np.sort(np.argsort(rng.random((n, L, E)), axis=2)[:, :, :K], axis=2).astype(np.uint8)


def test_append_then_gather_is_the_transpose_of_what_was_appended():
    L, K, E, P = 5, 4, 32, 16
    lens = [37, 16, 1, 50]
    tables, next_page = [], 0
    for n in lens:
        nb = (n + P - 1) // P
        tables.append(list(range(next_page, next_page + nb)) + [-1] * (4 - nb))
        next_page += nb
    # give the pages out in a scattered physical order: the table is the only link
    perm = np.random.default_rng(0).permutation(next_page)
    tables = [[int(perm[p]) if p >= 0 else -1 for p in t] for t in tables]
    pages = np.full((next_page, P, L, K), 255, np.uint8)
    per_seq = [_ids(n, L, K, E, 10 + s) for s, n in enumerate(lens)]
    # token by token, sequences interleaved, as decode steps would arrive
    for pos in range(max(lens)):
        live = [s for s, n in enumerate(lens) if pos < n]
        mc.append(pages, P, tables, live, [pos] * len(live), np.stack([per_seq[s][pos] for s in live]))
    start = np.concatenate([[0], np.cumsum(lens)])
    got = mc.gather(pages, P, tables, start)
    want = np.concatenate(per_seq, axis=0).transpose(1, 0, 2)         # [T,L,K] -> [L,T,K]
    assert np.array_equal(got, want)
    # slots past a sequence's end in its last page were never written
    last = tables[2][0]
    assert (pages[last, 1:] == 255).all()


def test_a_shared_prefix_is_the_same_pages_in_two_tables():
    """Multi-turn use: turn 2 continues turn 1.  Its table starts with turn 1's full pages; only the new
    tokens are appended; the gathered record of turn 2 begins with turn 1's record bit for bit."""
    L, K, E, P = 3, 8, 128, 8
    n1, n2 = 24, 24 + 13                                            # turn 1 ends on a page boundary
    ids = _ids(n2, L, K, E, 3)
    pages = np.zeros((8, P, L, K), np.uint8)
    t1 = [5, 2, 7, -1, -1]
    mc.append(pages, P, [t1], [0] * n1, list(range(n1)), ids[:n1])
    t2 = [5, 2, 7, 0, 4]                                            # same three pages, two new ones
    mc.append(pages, P, [t1, t2], [1] * (n2 - n1), list(range(n1, n2)), ids[n1:])
    r1 = mc.gather(pages, P, [t1], [0, n1])
    r2 = mc.gather(pages, P, [t2], [0, n2])
    assert np.array_equal(r2[:, :n1], r1) and np.array_equal(r2, ids.transpose(1, 0, 2))
    both = mc.gather(pages, P, [t1, t2], [0, n1, n1 + n2])           # packed batch of the two
    assert np.array_equal(both[:, :n1], r1) and np.array_equal(both[:, n1:], r2)


def test_page_size_one_and_empty_sequences():
    L, K, P = 2, 2, 1
    ids = _ids(3, L, K, 8, 1)
    pages = np.zeros((3, P, L, K), np.uint8)
    mc.append(pages, P, [[2, 0, 1]], [0, 0, 0], [0, 1, 2], ids)
    got = mc.gather(pages, P, [[-1, -1, -1], [2, 0, 1], [-1, -1, -1]], [0, 0, 3, 3])
    assert np.array_equal(got, ids.transpose(1, 0, 2))


def test_rollout_batch_layout_is_consistent():
    """The seeded batch layout the GPU tests and the bench use: lengths add up, every position has a page, a
    shared prefix is whole pages of the group's first sequence, and no page is owned twice."""
    from paper_2510_11370_amd import synth
    for T, P, group in ((1000, 16, 4), (131072, 16, 4), (65, 1, 4), (300, 8, 1), (5, 4, 4)):
        lens, shared, table, num_pages = synth.rollout_batch(T, P, group=group, seed=T)
        assert lens.sum() == T and (lens > 0).all() and (shared % P == 0).all() and (shared <= lens).all()
        owned = []
        owner = 0
        for s in range(len(lens)):
            nb = (lens[s] + P - 1) // P
            assert (table[s, :nb] >= 0).all() and (table[s, :nb] < num_pages).all() and (table[s, nb:] == -1).all()
            if shared[s] == 0:
                owner = s
            else:
                k = shared[s] // P
                assert np.array_equal(table[s, :k], table[owner, :k])
            owned.extend(table[s, shared[s] // P:nb].tolist())
        assert len(owned) == len(set(owned)) == num_pages
