"""r3_permute_static (the entry point that allocates nothing: its scratch is a fixed array inside the
library's device code) against r3_permute, through the C ABI: every output bit for bit, on two calls in a
row, the second with a smaller input (the array keeps the first call's contents)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2510_11370_amd import r3

pytestmark = pytest.mark.gpu


def _run(T, d, E, K, seed, stride_pad=0, with_rows=True):
    dev = "cuda"
    g = torch.Generator(device=dev).manual_seed(seed)
    idt = torch.uint8 if E <= 256 else torch.int32
    ids = torch.rand(T, E, generator=g, device=dev).argsort(dim=1)[:, :K].sort(dim=1).values
    stride = K + stride_pad
    rec = torch.zeros(T, stride, dtype=torch.int32, device=dev)
    rec[:, :K] = ids
    rec = rec.to(torch.uint8) if E <= 256 else rec.to(torch.uint16)
    D = r3.desc(T, d, E, K, 64, "bf16", idx_token_stride=stride if stride_pad else 0)
    x = torch.randn(T, d, generator=g, device=dev).to(torch.bfloat16)
    out = []
    for static in (False, True):
        o = dict(counts=torch.full((E,), -1, dtype=torch.int32, device=dev),
                 offsets=torch.full((E + 1,), -1, dtype=torch.int32, device=dev),
                 inv_perm=torch.full((T * K,), -1, dtype=torch.int32, device=dev),
                 perm=torch.full((T * K,), -1, dtype=torch.int32, device=dev),
                 Xp=torch.zeros(T * K, d, dtype=torch.bfloat16, device=dev) if with_rows else None,
                 status=torch.zeros(1, dtype=torch.int32, device=dev))
        if static:
            r3.permute_static(D, x, rec, o["counts"], o["offsets"], o["inv_perm"], o["perm"], o["Xp"], o["status"])
        else:
            ws = r3.workspace(D, r3.OP_PERMUTE)
            r3.permute(D, x, rec, o["counts"], o["offsets"], o["inv_perm"], o["perm"], o["Xp"], ws, o["status"])
        out.append(o)
    torch.cuda.synchronize()
    a, b = out
    for k in a:
        if a[k] is not None:
            assert torch.equal(a[k], b[k]), (k, T, E, K)
    assert int(b["status"].item()) == 0
    assert int(b["offsets"][-1].item()) == T * K and int(b["counts"].sum().item()) == T * K
    # a permutation: every row is named once
    assert torch.equal(torch.sort(b["perm"]).values, torch.arange(T * K, dtype=torch.int32, device=dev))


def test_static_scratch_permute_matches_the_workspace_call_twice_in_a_row():
    _run(T=16384, d=256, E=128, K=8, seed=1)          # 128 chunks of 1024 slots
    _run(T=1000, d=64, E=128, K=8, seed=2)            # smaller, ragged last chunk: scratch holds the first call's data
    _run(T=3001, d=32, E=640, K=6, seed=3, stride_pad=2, with_rows=False)   # uint16 ids, token stride, no row copy


def test_static_scratch_rejects_what_does_not_fit():
    big = r3.desc(131072, 64, 2048, 8, 64)            # 512 chunks * 2048 experts * 8 B = 8 MiB > 4 MiB
    assert r3.workspace_bytes(big, r3.OP_PERMUTE) > 4 << 20
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc = r3.lib().r3_permute_static(C.byref(big), None, C.c_void_p(one.data_ptr()), None, None, None, None, None,
                                    None, None)
    assert rc == 2                                      # R3_ERR_UNSUPPORTED, before any launch
