"""GPU parity of the router-mask cache (Section 4.2) against oracle/mask_cache.py: pure copies, so the page
pool and the gathered record are compared bit for bit, through the C ABI."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import mask_cache as mc
from paper_2510_11370_amd import r3, synth

pytestmark = pytest.mark.gpu


def _ids(n, L, K, E, rng, dt):
    """[n, L, K] ascending sets of distinct expert ids (plain random ids for very long sequences, where
    drawing distinct sets would dominate the test's time; a copy does not care)."""
    if n * L > 60000:
        return rng.integers(0, E, (n, L, K)).astype(dt)
    keys = rng.random((n, L, E), dtype=np.float32)
    return np.sort(np.argpartition(keys, K, axis=2)[:, :, :K], axis=2).astype(dt)


def _batch(T, L, K, E, P, seed, group=4):
    dt = np.uint8 if E <= 256 else np.uint16
    rng = np.random.default_rng(seed)
    lens, shared, table, num_pages = synth.rollout_batch(T, P, group=group, seed=seed)
    per_seq, owner = [], 0
    for s, n in enumerate(lens):
        ids = _ids(int(n), L, K, E, rng, dt)
        if shared[s] == 0:
            owner = s
        else:
            ids[:shared[s]] = per_seq[owner][:shared[s]]       # the common prompt has one set of masks
        per_seq.append(ids)
    return dt, lens, shared, table, num_pages, per_seq


def _append_all(pages_np, pages, table_np, table, P, lens, shared, per_seq, layer_major, status):
    """Every sequence appends the tokens it owns (everything after its shared pages) in one call each on
    the oracle and in one batched call on the GPU."""
    seq_id = np.concatenate([np.full(int(n - sh), s, np.int32) for s, (n, sh) in enumerate(zip(lens, shared))])
    pos = np.concatenate([np.arange(sh, n, dtype=np.int32) for n, sh in zip(lens, shared)])
    new = np.concatenate([ids[sh:] for ids, sh in zip(per_seq, shared)], axis=0)      # [n, L, K]
    mc.append(pages_np, P, table_np, seq_id, pos, new)
    n, L, K = new.shape
    if layer_major:
        src = torch.from_numpy(np.ascontiguousarray(new.transpose(1, 0, 2))).cuda()
        ls, ts = n * K, K
    else:
        src = torch.from_numpy(new).cuda()
        ls, ts = K, L * K
    r3.mask_cache_append(pages, table, torch.from_numpy(seq_id).cuda(), torch.from_numpy(pos).cuda(), src, ls, ts,
                         status)
    return n


@pytest.mark.parametrize("T,L,K,E,P,layer_major", [
    (1000, 5, 4, 32, 16, False),      # 4-byte units
    (1000, 48, 8, 128, 16, True),     # the paper's model: 8-byte units, source as L record_topk calls leave it
    (777, 94, 8, 384, 32, False),     # two-byte ids: 16-byte units, layers split over two chunks
    (300, 7, 3, 8, 4, True),          # odd K: byte units, three per router
    (300, 3, 6, 300, 8, False),       # 12-byte routers: 4-byte units, three per router
    (65, 2, 8, 128, 1, False),        # one token per page
    (1, 1, 1, 2, 16, False),
])
def test_append_and_gather_match_oracle(T, L, K, E, P, layer_major):
    dt, lens, shared, table_np, num_pages, per_seq = _batch(T, L, K, E, P, seed=T + L)
    tdt = torch.uint8 if dt == np.uint8 else torch.uint16
    fill = 201
    pages_np = np.full((num_pages, P, L, K), fill, dt)
    pages = torch.full((num_pages, P, L, K), fill, dtype=tdt, device="cuda")
    table = torch.from_numpy(table_np).cuda()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    _append_all(pages_np, pages, table_np, table, P, lens, shared, per_seq, layer_major, status)
    torch.cuda.synchronize()
    assert np.array_equal(pages.cpu().numpy(), pages_np)            # unwritten slots untouched
    start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    out = torch.full((L, T, K), 77, dtype=tdt, device="cuda")
    r3.mask_cache_gather(pages, table, torch.from_numpy(start).cuda(), out, status)
    torch.cuda.synchronize()
    want = mc.gather(pages_np, P, table_np, start)
    assert np.array_equal(out.cpu().numpy(), want)
    # and what the batch was built from, directly: the transpose of every sequence's own ids
    assert np.array_equal(want, np.concatenate(per_seq, axis=0).transpose(1, 0, 2))
    assert int(status.item()) == 0
    assert T < 1000 or (shared > 0).any()


def test_full_size_stack_record():
    """The 48-layer, 131072-token batch: gathered record against the oracle in full."""
    sh = synth.CONFIGS["stack48_128k"]
    T, L, K, E, P = sh.T, sh.layers, sh.K, sh.E, 16
    dt, lens, shared, table_np, num_pages, per_seq = _batch(T, L, K, E, P, seed=9)
    pages_np = np.zeros((num_pages, P, L, K), dt)
    pages = torch.zeros((num_pages, P, L, K), dtype=torch.uint8, device="cuda")
    table = torch.from_numpy(table_np).cuda()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    _append_all(pages_np, pages, table_np, table, P, lens, shared, per_seq, True, status)
    start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    out = torch.empty((L, T, K), dtype=torch.uint8, device="cuda")
    r3.mask_cache_gather(pages, table, torch.from_numpy(start).cuda(), out, status)
    torch.cuda.synchronize()
    assert np.array_equal(pages.cpu().numpy(), pages_np)
    assert np.array_equal(out.cpu().numpy(), mc.gather(pages_np, P, table_np, start))
    assert int(status.item()) == 0 and shared.sum() > 0


def test_decode_steps_then_second_turn():
    """Token-by-token appends of interleaved sequences (decode steps), then a second turn that reuses the
    first turn's pages as its prefix and appends only its own tokens."""
    L, K, E, P = 6, 8, 128, 8
    rng = np.random.default_rng(4)
    lens1 = [24, 9, 40]
    ids1 = [_ids(n, L, K, E, rng, np.uint8) for n in lens1]
    table_np = -np.ones((6, 10), np.int32)
    pool = list(rng.permutation(40))
    for s, n in enumerate(lens1):
        for b in range((n + P - 1) // P):
            table_np[s, b] = pool.pop()
    pages_np = np.zeros((40, P, L, K), np.uint8)
    pages = torch.zeros((40, P, L, K), dtype=torch.uint8, device="cuda")
    table = torch.from_numpy(table_np).cuda()
    for pos in range(max(lens1)):
        live = np.array([s for s, n in enumerate(lens1) if pos < n], np.int32)
        new = np.stack([ids1[s][pos] for s in live])
        mc.append(pages_np, P, table_np, live, np.full(len(live), pos, np.int32), new)
        r3.mask_cache_append(pages, table, torch.from_numpy(live).cuda(),
                             torch.full((len(live),), pos, dtype=torch.int32, device="cuda"),
                             torch.from_numpy(new).cuda(), K, L * K)
    # second turn: sequences 3, 4 continue 0 and 2 (page-aligned length 24 and 40), 5 is new
    ext = {3: (0, 24, 11), 4: (2, 40, 30), 5: (None, 0, 5)}
    ids2 = {}
    for s, (src, keep, extra) in ext.items():
        if src is not None:
            table_np[s, :keep // P] = table_np[src, :keep // P]
        for b in range(keep // P, (keep + extra + P - 1) // P):
            table_np[s, b] = pool.pop()
        ids2[s] = _ids(extra, L, K, E, rng, np.uint8)
    table = torch.from_numpy(table_np).cuda()
    seq_id = np.concatenate([np.full(e, s, np.int32) for s, (_, k, e) in ext.items()])
    pos = np.concatenate([np.arange(k, k + e, dtype=np.int32) for s, (_, k, e) in ext.items()])
    new = np.concatenate([ids2[s] for s in ext])
    mc.append(pages_np, P, table_np, seq_id, pos, new)
    r3.mask_cache_append(pages, table, torch.from_numpy(seq_id).cuda(), torch.from_numpy(pos).cuda(),
                         torch.from_numpy(new).cuda(), K, L * K)
    lens = lens1 + [k + e for (_, k, e) in ext.values()]
    start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    out = torch.empty((L, int(start[-1]), K), dtype=torch.uint8, device="cuda")
    r3.mask_cache_gather(pages, table, torch.from_numpy(start).cuda(), out)
    torch.cuda.synchronize()
    assert np.array_equal(pages.cpu().numpy(), pages_np)
    got = out.cpu().numpy()
    assert np.array_equal(got, mc.gather(pages_np, P, table_np, start))
    full3 = np.concatenate([ids1[0], ids2[3]]).transpose(1, 0, 2)
    assert np.array_equal(got[:, start[3]:start[4]], full3)          # turn 2 of sequence 0: prefix + new tokens


def test_gathered_record_replays_like_the_direct_one():
    """Record with r3_record_topk per layer into [L][n][K], store, gather: the gathered record is the
    recorded one, so every consumer of idx sees the same bytes."""
    L, T, E, K, P = 4, 1500, 128, 8, 16
    lens, shared, table_np, num_pages = synth.rollout_batch(T, P, group=1, seed=5)
    D = r3.desc(T, 64, E, K, 64)
    g = torch.Generator(device="cuda").manual_seed(11)
    rec = torch.zeros(L, T, K, dtype=torch.uint8, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    for l in range(L):
        r3.record_topk(D, torch.randn(T, E, device="cuda", generator=g), rec[l], status)
    start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    seq_id = np.repeat(np.arange(len(lens), dtype=np.int32), lens)
    pos = (np.arange(T) - start[seq_id]).astype(np.int32)
    pages = torch.zeros((num_pages, P, L, K), dtype=torch.uint8, device="cuda")
    table = torch.from_numpy(table_np).cuda()
    r3.mask_cache_append(pages, table, torch.from_numpy(seq_id).cuda(), torch.from_numpy(pos).cuda(), rec, T * K, K,
                         status)
    out = torch.zeros_like(rec)
    r3.mask_cache_gather(pages, table, torch.from_numpy(start).cuda(), out, status)
    torch.cuda.synchronize()
    assert torch.equal(out, rec) and int(status.item()) == 0


def test_bad_addresses_are_flagged_and_touch_nothing():
    L, K, P = 3, 8, 4
    pages = torch.full((5, P, L, K), 9, dtype=torch.uint8, device="cuda")
    table = torch.tensor([[0, 1, -1], [2, 7, 3]], dtype=torch.int32, device="cuda")     # page 7 does not exist
    new = torch.arange(6 * L * K, dtype=torch.uint8, device="cuda").reshape(6, L, K)
    seq_id = torch.tensor([0, 0, 1, 2, -1, 1], dtype=torch.int32, device="cuda")
    pos = torch.tensor([1, 9, 5, 0, 0, 12], dtype=torch.int32, device="cuda")
    #            ok, block 2 unset, page 7, seq 2, seq -1, block 3 past the table
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    r3.mask_cache_append(pages, table, seq_id, pos, new, K, L * K, status)
    torch.cuda.synchronize()
    want = np.full((5, P, L, K), 9, np.uint8)
    want[0, 1] = new[0].cpu().numpy()
    assert np.array_equal(pages.cpu().numpy(), want) and int(status.item()) == 8
    # gather: sequence 0 has 6 tokens (block 1 valid), sequence 1 has 7 (tokens 4..6 on the missing page)
    status.zero_()
    start = torch.tensor([0, 6, 13], dtype=torch.int32, device="cuda")
    out = torch.full((L, 13, K), 5, dtype=torch.uint8, device="cuda")
    r3.mask_cache_gather(pages, table, start, out, status)
    torch.cuda.synchronize()
    ref = mc.gather(np.concatenate([want, np.zeros((3, P, L, K), np.uint8)]), P,
                    np.array([[0, 1, -1], [2, 5, 3]]), [0, 6, 13])                 # page 5 of the padded pool: zeros
    assert np.array_equal(out.cpu().numpy(), ref) and int(status.item()) == 8


def test_empty_inputs_and_host_errors():
    lib = r3.lib()
    L, K, P = 2, 8, 4
    pages = torch.zeros((2, P, L, K), dtype=torch.uint8, device="cuda")
    table = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    i32 = torch.zeros(4, dtype=torch.int32, device="cuda")
    out = torch.full((L, 4, K), 3, dtype=torch.uint8, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    ap = lambda **kw: lib.r3_mask_cache_append(
        C.c_int(kw.get("dt", 0)), C.c_int(kw.get("L", L)), C.c_int(K), C.c_int(kw.get("P", P)),
        kw.get("pages", p(pages)), C.c_int64(2), p(table), C.c_int(1), C.c_int(2), C.c_int64(kw.get("n", 0)),
        kw.get("seq", p(i32)), p(i32), p(out), C.c_int64(K), C.c_int64(L * K), None, None)
    ga = lambda **kw: lib.r3_mask_cache_gather(
        C.c_int(kw.get("dt", 0)), C.c_int(L), C.c_int(K), C.c_int(P), p(pages), C.c_int64(kw.get("np_", 2)),
        p(table), C.c_int(kw.get("nseq", 1)), C.c_int(2), kw.get("start", p(i32)), C.c_int64(kw.get("T", 0)),
        kw.get("out", p(out)), None, None)
    assert ap() == 0 and ga() == 0                                   # n = 0, T = 0: nothing to do
    torch.cuda.synchronize()
    assert (out == 3).all() and not pages.any()
    assert ap(dt=2) == 1 and ap(L=0) == 1 and ap(P=0) == 1 and ap(pages=None) == 1 and ap(n=-1) == 1
    assert ap(n=1, seq=None) == 1
    assert ga(dt=5) == 1 and ga(np_=0) == 1 and ga(nseq=0) == 1 and ga(start=None) == 1 and ga(T=-1) == 1
    assert ga(T=4, out=None) == 1
    # empty sequences inside a batch
    pages[0, :3] = torch.arange(3 * L * K, dtype=torch.uint8, device="cuda").reshape(3, L, K)
    table2 = torch.tensor([[-1, -1], [0, -1], [-1, -1]], dtype=torch.int32, device="cuda")
    start = torch.tensor([0, 0, 3, 3], dtype=torch.int32, device="cuda")
    out3 = torch.zeros((L, 3, K), dtype=torch.uint8, device="cuda")
    r3.mask_cache_gather(pages, table2, start, out3)
    torch.cuda.synchronize()
    assert torch.equal(out3, pages[0, :3].permute(1, 0, 2))
