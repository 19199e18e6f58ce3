"""kvc_compress under HIP graph capture: the library enqueues kernels only (no
allocation, no memset, no host synchronisation), so a call can be recorded once and
replayed; every replay must reproduce the eager call bit for bit, also with the
program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import paper_2509_05165_amd as kv
import workloads as wl
from kvc_testlib import DeviceWorkload, Workload

pytestmark = pytest.mark.gpu


def _call(dw, p, outs, stream):
    w = dw.w
    kv.kvc_compress(p, dw.ptrs(dw.q), dw.ptrs(dw.k), dw.ptrs(dw.v), w.cu, w.budgets,
                    outs["k_out"].data_ptr(), outs["v_out"].data_ptr(), outs["lengths"].data_ptr(),
                    outs["offsets"].data_ptr(), dw.ws.data_ptr(), dw.ws_bytes, stream,
                    tau=outs["tau"].data_ptr())


@pytest.mark.parametrize("lens", [[1500, 700], [9000]])
def test_compress_replays_from_a_graph(lens):
    print(f"[case] graph capture lens={lens}", flush=True)
    cfg = wl.get_config(5, batch=len(lens), layers=3)
    w = Workload(cfg, seed=21, lens=lens)
    dw = DeviceWorkload(w)
    p = w.params()
    tb, c = sum(w.budgets), cfg

    def fresh():
        return {"k_out": torch.zeros(tb * c.hkv * c.head_dim, dtype=torch.bfloat16, device="cuda"),
                "v_out": torch.zeros(tb * c.hkv * c.head_dim, dtype=torch.bfloat16, device="cuda"),
                "lengths": torch.full((c.batch * c.layers,), -1, dtype=torch.int32, device="cuda"),
                "offsets": torch.full((c.batch * c.layers + 1,), -1, dtype=torch.int64, device="cuda"),
                "tau": torch.zeros(c.batch, dtype=torch.float32, device="cuda")}

    eager = fresh()
    _call(dw, p, eager, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert int(eager["lengths"].sum()) == tb

    outs = fresh()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _call(dw, p, outs, torch.cuda.current_stream().cuda_stream)
    for replay in range(3):
        for t in outs.values():                      # eager work between the replays
            t.fill_(7)
        dw.ws.fill_(0xAB)                            # the workspace holds nothing a replay relies on
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in outs:
            a, b = outs[name], eager[name]
            if a.dtype == torch.bfloat16:
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), (replay, name)
