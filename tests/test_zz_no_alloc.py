"""kvc_global_select_static (the entry point that allocates nothing: its
histograms, counters and tickets live in a buffer inside the library's device
image) against kvc_global_select on the same inputs, through the C ABI: tau,
lengths and offsets must be bit-identical.  Two calls in a row share the
buffer, the second on a smaller problem, so stale contents of the first would
show."""
import numpy as np
import pytest
import torch

import paper_2509_05165_amd as kv
from kvc_testlib import stream, to_dev

pytestmark = pytest.mark.gpu


def _pool(lyr, lens, kind, seed):
    r = np.random.default_rng([4242, seed])
    total = int(sum(lens))
    if kind == "smooth":
        i_all = np.exp(r.standard_normal((lyr, total)) * 2 - 9)
    else:   # many ties at the threshold
        i_all = np.round(r.random((lyr, total)) * 6) / 8
    i_all = i_all.astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    for b in range(len(lens)):     # each row non-increasing inside a sequence
        lo, hi = int(cu[b]), int(cu[b + 1])
        i_all[:, lo:hi] = -np.sort(-i_all[:, lo:hi], axis=1)
    return i_all, cu


def _both(lyr, lens, fracs, kind, seed, **pkw):
    i_all, cu = _pool(lyr, lens, kind, seed)
    budgets = [int(f * lyr * n) for f, n in zip(fracs, lens)]
    p = kv.KvcParams(len(lens), lyr, 8, 8, 128, 64, kv.KVC_BF16, **pkw)
    total = int(cu[-1])
    ws_bytes = kv.kvc_workspace_size(p, total, max(lens))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    I = to_dev(i_all)
    out = []
    for static in (False, True):
        tau = torch.full((len(lens),), -7.0, dtype=torch.float32, device="cuda")
        lengths = torch.full((len(lens) * lyr,), -1, dtype=torch.int32, device="cuda")
        offsets = torch.full((len(lens) * lyr + 1,), -1, dtype=torch.int64, device="cuda")
        if static:
            kv.kvc_global_select_static(p, I.data_ptr(), cu, budgets, tau.data_ptr(),
                                        lengths.data_ptr(), offsets.data_ptr(), stream())
        else:
            kv.kvc_global_select(p, I.data_ptr(), cu, budgets, tau.data_ptr(), lengths.data_ptr(),
                                 offsets.data_ptr(), ws.data_ptr(), ws_bytes, stream())
        torch.cuda.synchronize()
        out.append((tau.cpu().numpy(), lengths.cpu().numpy(), offsets.cpu().numpy()))
    (t0, l0, o0), (t1, l1, o1) = out
    np.testing.assert_array_equal(t0.view(np.uint32), t1.view(np.uint32))
    np.testing.assert_array_equal(l0, l1)
    np.testing.assert_array_equal(o0, o1)
    assert int(l1.sum()) == sum(budgets) and o1[-1] == sum(budgets)


@pytest.mark.parametrize("kind", ["smooth", "ties"])
def test_static_select_matches_workspace_select_twice(kind):
    print(f"[case] static select {kind}: big then small", flush=True)
    # first a pool of 32 rows x (70000 + 3000) tokens in two sequences, then a
    # much smaller one (fewer rows, fewer sequences, fewer workgroups)
    _both(32, [70000, 3000], [0.15, 0.5], kind, 1)
    _both(3, [777], [0.3], kind, 2)
    # once more with a per-row floor, then a zero budget beside a full one
    _both(5, [3000, 1, 500], [0.4, 1.0, 0.2], kind, 3, min_per_layer=2)
    _both(4, [900, 40], [0.0, 1.0], kind, 4)
