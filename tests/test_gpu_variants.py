"""GPU parity of the variants (value-norm weighting, per-layer floor, position
order, unstructured selection) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2509_05165_amd as kv
import workloads as wl
from oracle import kvc_oracle as orc
from kvc_testlib import DeviceWorkload, Workload, stream, to_dev, to_host_bits, EPS
from test_gpu_parity import _select_case

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)


# ------------------------------------------------------------- value norm
VNORM_CASES = {
    "tiny-f32": (0, dict(layers=2), {}),
    "f32-ragged-d20": (0, dict(layers=1, hq=6, hkv=2, n=777, window=20, head_dim=20), {}),
    "bf16-mfma": (1, dict(layers=2, n=1500), {}),
    "bf16-mfma-mean-max": (1, dict(layers=1, n=900), dict(agg_task=kv.KVC_AGG_MEAN, agg_group=kv.KVC_AGG_MAX)),
    "bf16-gqa8-m128-rowchunks": (4, dict(layers=1, n=700), {}),
    "bf16-12-kv-heads": (1, dict(layers=1, hq=24, hkv=12, n=300), dict(add_head_mean=0)),
    "bf16-varlen-batch": (3, dict(layers=1, batch=3, n_range=(200, 900)), {}),
}


@pytest.mark.parametrize("name", list(VNORM_CASES))
def test_value_norm_scores_match_oracle(name):
    cid, over, pkw = VNORM_CASES[name]
    _say(f"vnorm {name}")
    cfg = wl.get_config(cid, **over)
    w = Workload(cfg)
    # value rows with norms spread over two orders of magnitude, as the appendix reports
    r = np.random.default_rng(17)
    for l in range(cfg.layers):
        scale = np.exp(r.uniform(np.log(0.1), np.log(10.0), size=w.v[l].shape[:2] + (1,)))
        if w.v[l].dtype == np.uint16:
            f = (w.v[l].astype(np.uint32) << 16).view(np.float32) * scale.astype(np.float32)
            w.v[l] = wl.f32_to_bf16_bits(f)
        else:
            w.v[l] = (w.v[l] * scale).astype(np.float32)
    dw = DeviceWorkload(w)
    p = w.params(value_norm=1, **pkw)
    ws_bytes = kv.kvc_workspace_size(p, w.total, int(w.lens.max()))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    S = torch.zeros((cfg.layers, cfg.hkv, w.total), dtype=torch.float32, device="cuda")
    kv.kvc_score(p, dw.ptrs(dw.q), dw.ptrs(dw.k), w.cu, S.data_ptr(), ws.data_ptr(), ws_bytes,
                 stream(), v=dw.ptrs(dw.v))
    torch.cuda.synchronize()
    got = S.cpu().numpy()
    okw = dict(agg_task=pkw.get("agg_task", orc.AGG_MAX), agg_group=pkw.get("agg_group", orc.AGG_MEAN),
               add_head_mean=bool(pkw.get("add_head_mean", 1)))
    worst = 0.0
    for b in range(cfg.batch):
        lo, hi = int(w.cu[b]), int(w.cu[b + 1])
        for l in range(cfg.layers):
            q = orc.widen(w.q[l][b])
            ref = orc.score_layer(q, orc.widen(w.k[l][:, lo:hi]), v=orc.widen(w.v[l][:, lo:hi]), **okw)
            np.testing.assert_allclose(got[l][:, lo:hi], ref, rtol=EPS, atol=0)
            worst = max(worst, float(np.max(np.abs(got[l][:, lo:hi] - ref) / ref)))
    assert worst < 1e-4, worst          # fp32 pipeline: far inside the tolerance


# ------------------------------------------------------------ per-layer floor
@pytest.mark.parametrize("kind", ["smooth", "ties", "equal-layers"])
@pytest.mark.parametrize("lyr,lens,fracs,floor", [
    (4, [1024], [0.25], 3), (3, [5000], [0.5], 2500), (5, [3000, 1, 777], [0.2, 1.0, 0.5], 2),
    (32, [4096], [0.1], 100), (2, [2049, 2048], [0.999, 0.3], 600), (3, [40], [0.5], 1000)])
def test_global_select_floor_bit_exact(kind, lyr, lens, fracs, floor):
    _say(f"select floor {kind} lyr={lyr} lens={lens} fracs={fracs} floor={floor}")
    i_all, cu = _select_case(lyr, lens, fracs, kind, lyr)
    budgets = [max(int(f * lyr * n), lyr * min(floor, n)) for f, n in zip(fracs, lens)]
    total = int(cu[-1])
    p = kv.KvcParams(len(lens), lyr, 8, 8, 128, 64, kv.KVC_BF16, min_per_layer=floor)
    ws_bytes = kv.kvc_workspace_size(p, total, max(lens))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    I = to_dev(i_all)
    tau = torch.zeros(len(lens), dtype=torch.float32, device="cuda")
    lengths = torch.full((len(lens) * lyr,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((len(lens) * lyr + 1,), -1, dtype=torch.int64, device="cuda")
    kv.kvc_global_select(p, I.data_ptr(), cu, budgets, tau.data_ptr(), lengths.data_ptr(),
                         offsets.data_ptr(), ws.data_ptr(), ws_bytes, stream())
    torch.cuda.synchronize()
    gl = lengths.cpu().numpy().reshape(len(lens), lyr)
    gt = tau.cpu().numpy()
    for b in range(len(lens)):
        lo, hi = int(cu[b]), int(cu[b + 1])
        rl, rt = orc.global_select(i_all[:, lo:hi].astype(np.float64), budgets[b], floor)
        np.testing.assert_array_equal(gl[b], rl)
        if rt is not None:
            assert np.float32(rt) == gt[b]
        else:
            assert np.isinf(gt[b]) and gt[b] > 0
    go = offsets.cpu().numpy()
    np.testing.assert_array_equal(go, np.concatenate([[0], np.cumsum(gl.reshape(-1))]))


# --------------------------------------------------- unstructured selection
@pytest.mark.parametrize("kind", ["smooth", "ties"])
@pytest.mark.parametrize("floor", [0, 5])
@pytest.mark.parametrize("lyr,hkv", [(3, 4), (75, 8)])      # 600 rows: several chunks of the bookkeeping scan
def test_unstructured_select_bit_exact(kind, floor, lyr, hkv):
    lens, fracs = [1500, 70], [0.3, 0.6]
    _say(f"unstructured select {kind} floor={floor} rows={lyr * hkv}")
    rows = lyr * hkv
    s_sorted, cu = _select_case(rows, lens, fracs, kind, 7)          # rows = (layer, head)
    budgets = [max(int(f * rows * n), rows * min(floor, n)) for f, n in zip(fracs, lens)]
    total = int(cu[-1])
    p = kv.KvcParams(len(lens), lyr, hkv, hkv, 128, 64, kv.KVC_BF16, unstructured=1, min_per_layer=floor)
    ws_bytes = kv.kvc_workspace_size(p, total, max(lens))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    ss = to_dev(s_sorted)
    tau = torch.zeros(len(lens), dtype=torch.float32, device="cuda")
    lengths = torch.full((len(lens) * rows,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((len(lens) * rows + 1,), -1, dtype=torch.int64, device="cuda")
    kv.kvc_global_select(p, ss.data_ptr(), cu, budgets, tau.data_ptr(), lengths.data_ptr(),
                         offsets.data_ptr(), ws.data_ptr(), ws_bytes, stream())
    torch.cuda.synchronize()
    gl = lengths.cpu().numpy().reshape(len(lens), rows)
    for b in range(len(lens)):
        lo, hi = int(cu[b]), int(cu[b + 1])
        rl, rt = orc.global_select(s_sorted[:, lo:hi].astype(np.float64), budgets[b], floor)
        np.testing.assert_array_equal(gl[b], rl)
        assert np.float32(rt) == tau.cpu().numpy()[b]
    np.testing.assert_array_equal(offsets.cpu().numpy(), np.concatenate([[0], np.cumsum(gl.reshape(-1))]))


def _gather_inputs(r, dtype, d, lyr, hkv, lens):
    cu = np.concatenate([[0], np.cumsum(lens)])
    total = int(cu[-1])
    if dtype == "bf16":
        ks = [r.integers(0, 2 ** 16, size=(hkv, total, d)).astype(np.uint16) for _ in range(lyr)]
        vs = [r.integers(0, 2 ** 16, size=(hkv, total, d)).astype(np.uint16) for _ in range(lyr)]
    else:
        ks = [r.standard_normal((hkv, total, d)).astype(np.float32) for _ in range(lyr)]
        vs = [r.standard_normal((hkv, total, d)).astype(np.float32) for _ in range(lyr)]
    idx = np.zeros((lyr, hkv, total), dtype=np.int32)
    for l in range(lyr):
        for h in range(hkv):
            for b in range(len(lens)):
                idx[l, h, cu[b]:cu[b + 1]] = r.permutation(lens[b])
    return cu, total, ks, vs, idx


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 20)])
@pytest.mark.parametrize("order", [kv.KVC_ORDER_RANK, kv.KVC_ORDER_POSITION])
def test_unstructured_gather_bit_exact(dtype, d, order):
    _say(f"unstructured gather {dtype} d={d} order={order}")
    r = np.random.default_rng(21)
    lyr, hkv, lens = 2, 3, [700, 33]
    cu, total, ks, vs, idx = _gather_inputs(r, dtype, d, lyr, hkv, lens)
    lengths = np.array([[[300, 0, 700], [1, 699, 64]], [[33, 5, 0], [0, 0, 32]]], dtype=np.int32)  # [b][l][h]
    offsets = np.concatenate([[0], np.cumsum(lengths.reshape(-1))]).astype(np.int64)
    tb = int(offsets[-1])
    p = kv.KvcParams(2, lyr, hkv, hkv, d, 64, kv.KVC_BF16 if dtype == "bf16" else kv.KVC_F32,
                     unstructured=1, order=order)
    ws_bytes = kv.kvc_workspace_size(p, total, max(lens))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    dk, dv = [to_dev(x) for x in ks], [to_dev(x) for x in vs]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    k_out = torch.zeros(tb * d, dtype=tdt, device="cuda")
    v_out = torch.zeros_like(k_out)
    d_idx, d_len, d_off = to_dev(idx), to_dev(lengths.reshape(-1)), to_dev(offsets)
    kv.kvc_gather(p, [t.data_ptr() for t in dk], [t.data_ptr() for t in dv], d_idx.data_ptr(),
                  d_len.data_ptr(), d_off.data_ptr(), cu, tb, k_out.data_ptr(), v_out.data_ptr(),
                  stream(), workspace=ws.data_ptr(), workspace_bytes=ws_bytes)
    torch.cuda.synchronize()
    gk, gv = to_host_bits(k_out), to_host_bits(v_out)
    for b in range(2):
        lo, hi = int(cu[b]), int(cu[b + 1])
        for l in range(lyr):
            rk = orc.gather_heads(ks[l][:, lo:hi], idx[l, :, lo:hi], lengths[b, l], order == kv.KVC_ORDER_POSITION)
            rv = orc.gather_heads(vs[l][:, lo:hi], idx[l, :, lo:hi], lengths[b, l], order == kv.KVC_ORDER_POSITION)
            for h in range(hkv):
                n = int(lengths[b, l, h])
                base = int(offsets[(b * lyr + l) * hkv + h]) * d
                np.testing.assert_array_equal(gk[base: base + n * d].reshape(n, d), rk[h])
                np.testing.assert_array_equal(gv[base: base + n * d].reshape(n, d), rv[h])


# ------------------------------------------------------------- position order
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
@pytest.mark.parametrize("lens", [[700, 33], [31], [4097, 1, 64]])
def test_position_order_gather_bit_exact(dtype, d, lens):
    _say(f"position gather {dtype} d={d} lens={lens}")
    r = np.random.default_rng(23)
    lyr, hkv = 3, 4
    cu, total, ks, vs, idx = _gather_inputs(r, dtype, d, lyr, hkv, lens)
    lengths = np.stack([r.integers(0, n + 1, size=lyr) for n in lens]).astype(np.int32)   # [b][l]
    lengths[0, 0] = lens[0]                    # one full block: must come back as the identity
    lengths[-1, -1] = 0
    offsets = np.concatenate([[0], np.cumsum(lengths.reshape(-1))]).astype(np.int64)
    tb = int(offsets[-1])
    nb = len(lens)
    p = kv.KvcParams(nb, lyr, hkv, hkv, d, 64, kv.KVC_BF16 if dtype == "bf16" else kv.KVC_F32,
                     order=kv.KVC_ORDER_POSITION)
    ws_bytes = kv.kvc_workspace_size(p, total, max(lens))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    ws.fill_(0xAB)                             # the stage must not rely on a clean workspace
    dk, dv = [to_dev(x) for x in ks], [to_dev(x) for x in vs]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    k_out = torch.zeros(max(tb, 1) * hkv * d, dtype=tdt, device="cuda")
    v_out = torch.zeros_like(k_out)
    d_idx, d_len, d_off = to_dev(idx), to_dev(lengths.reshape(-1)), to_dev(offsets)
    kv.kvc_gather(p, [t.data_ptr() for t in dk], [t.data_ptr() for t in dv], d_idx.data_ptr(),
                  d_len.data_ptr(), d_off.data_ptr(), cu, tb, k_out.data_ptr(), v_out.data_ptr(),
                  stream(), workspace=ws.data_ptr(), workspace_bytes=ws_bytes)
    torch.cuda.synchronize()
    gk, gv = to_host_bits(k_out), to_host_bits(v_out)
    for b in range(nb):
        lo, hi = int(cu[b]), int(cu[b + 1])
        for l in range(lyr):
            n = int(lengths[b, l])
            base = int(offsets[b * lyr + l]) * hkv * d
            rk = orc.gather(ks[l][:, lo:hi], idx[l, :, lo:hi], n, position_order=True)
            rv = orc.gather(vs[l][:, lo:hi], idx[l, :, lo:hi], n, position_order=True)
            np.testing.assert_array_equal(gk[base: base + hkv * n * d].reshape(hkv, n, d), rk)
            np.testing.assert_array_equal(gv[base: base + hkv * n * d].reshape(hkv, n, d), rv)
    np.testing.assert_array_equal(gk[: hkv * lens[0] * d].reshape(hkv, lens[0], d), ks[0][:, :lens[0]])


# ------------------------------------------------------------------ whole pass
def _run_variant(w, dw, **pkw):
    c = w.cfg
    p = w.params(**pkw)
    rows = c.layers * (c.hkv if pkw.get("unstructured") else 1)
    tb = sum(w.budgets)
    hpb = 1 if pkw.get("unstructured") else c.hkv
    tdtype = torch.bfloat16 if c.dtype == "bf16" else torch.float32
    ws_bytes = kv.kvc_workspace_size(p, w.total, int(w.lens.max()))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    k_out = torch.zeros(max(tb, 1) * hpb * c.head_dim, dtype=tdtype, device="cuda")
    v_out = torch.zeros_like(k_out)
    lengths = torch.full((c.batch * rows,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((c.batch * rows + 1,), -1, dtype=torch.int64, device="cuda")
    S = torch.zeros((c.layers, c.hkv, w.total), dtype=torch.float32, device="cuda")
    idx = torch.zeros((c.layers, c.hkv, w.total), dtype=torch.int32, device="cuda")
    ss = torch.zeros_like(S)
    tau = torch.zeros(c.batch, dtype=torch.float32, device="cuda")
    kv.kvc_compress(p, dw.ptrs(dw.q), dw.ptrs(dw.k), dw.ptrs(dw.v), w.cu, w.budgets,
                    k_out.data_ptr(), v_out.data_ptr(), lengths.data_ptr(), offsets.data_ptr(),
                    ws.data_ptr(), ws_bytes, stream(), scores=S.data_ptr(), idx=idx.data_ptr(),
                    s_sorted=ss.data_ptr(), tau=tau.data_ptr())
    torch.cuda.synchronize()
    return dict(S=S.cpu().numpy(), idx=idx.cpu().numpy(), S_sorted=ss.cpu().numpy(),
                lengths=lengths.cpu().numpy().reshape(c.batch, rows), offsets=offsets.cpu().numpy(),
                k_out=to_host_bits(k_out), v_out=to_host_bits(v_out), tau=tau.cpu().numpy())


def test_compress_position_order_full_budget_is_identity():
    cfg = wl.get_config(1, layers=2, n=1300, keep_percent=100)
    w = Workload(cfg)
    dw = DeviceWorkload(w)
    got = _run_variant(w, dw, order=kv.KVC_ORDER_POSITION)
    c = cfg
    assert got["lengths"].tolist() == [[1300, 1300]]
    for l in range(c.layers):
        base = l * 1300 * c.hkv * c.head_dim
        blk = got["k_out"][base: base + c.hkv * 1300 * c.head_dim].reshape(c.hkv, 1300, c.head_dim)
        np.testing.assert_array_equal(blk, w.k[l])
        blk = got["v_out"][base: base + c.hkv * 1300 * c.head_dim].reshape(c.hkv, 1300, c.head_dim)
        np.testing.assert_array_equal(blk, w.v[l])


@pytest.mark.parametrize("pkw", [dict(order=kv.KVC_ORDER_POSITION, min_per_layer=40),
                                 dict(value_norm=1), dict(min_per_layer=200)])
def test_compress_variants_end_to_end(pkw):
    """Lengths within the near-threshold band of the oracle, sum exact; rows are bit
    copies of what the GPU's own idx names, in the requested order."""
    _say(f"e2e variant {pkw}")
    cfg = wl.get_config(1, layers=3, n=2000)
    w = Workload(cfg)
    dw = DeviceWorkload(w)
    got = _run_variant(w, dw, **pkw)
    ref = w.oracle(value_norm=bool(pkw.get("value_norm")), position_order=pkw.get("order") == 1,
                   min_per_layer=pkw.get("min_per_layer", 0))[0]
    c, n, B = cfg, 2000, w.budgets[0]
    floor = pkw.get("min_per_layer", 0)
    np.testing.assert_allclose(got["S"], ref["S"], rtol=EPS)
    lens = got["lengths"][0]
    assert int(lens.sum()) == B and int(lens.min()) >= min(floor, n)
    tau = ref["tau"]
    for l in range(c.layers):
        nl = int(lens[l])
        comp = ref["I"][l][floor:]                        # entries that compete
        lo_ok = floor + int((comp > tau * (1 + EPS)).sum())
        hi_ok = floor + int((comp >= tau * (1 - EPS)).sum())
        assert lo_ok <= nl <= hi_ok
        base = int(got["offsets"][l]) * c.hkv * c.head_dim
        kblk = got["k_out"][base: base + c.hkv * nl * c.head_dim].reshape(c.hkv, nl, c.head_dim)
        vblk = got["v_out"][base: base + c.hkv * nl * c.head_dim].reshape(c.hkv, nl, c.head_dim)
        for h in range(c.hkv):
            rows = got["idx"][l, h, :nl]
            if pkw.get("order") == 1:
                rows = np.sort(rows)
            np.testing.assert_array_equal(kblk[h], w.k[l][h, rows])
            np.testing.assert_array_equal(vblk[h], w.v[l][h, rows])


def test_compress_unstructured_end_to_end():
    cfg = wl.get_config(1, layers=3, n=1800)
    w = Workload(cfg)
    rows = cfg.layers * cfg.hkv
    w.budgets = [rows * 1800 // 8]                        # budget counts (head, token) entries
    dw = DeviceWorkload(w)
    got = _run_variant(w, dw, unstructured=1)
    ref = w.oracle(unstructured=True)[0]
    c, n, B = cfg, 1800, w.budgets[0]
    np.testing.assert_allclose(got["S"], ref["S"], rtol=EPS)
    lens = got["lengths"][0].reshape(c.layers, c.hkv)
    assert int(lens.sum()) == B
    tau = ref["tau"]
    for l in range(c.layers):
        for h in range(c.hkv):
            nl = int(lens[l, h])
            srow = ref["S_sorted"][l, h]
            assert int((srow > tau * (1 + EPS)).sum()) <= nl <= int((srow >= tau * (1 - EPS)).sum())
            base = int(got["offsets"][l * c.hkv + h]) * c.head_dim
            kblk = got["k_out"][base: base + nl * c.head_dim].reshape(nl, c.head_dim)
            vblk = got["v_out"][base: base + nl * c.head_dim].reshape(nl, c.head_dim)
            sel = got["idx"][l, h, :nl]
            np.testing.assert_array_equal(kblk, w.k[l][h, sel])
            np.testing.assert_array_equal(vblk, w.v[l][h, sel])
            chosen = np.zeros(n, dtype=bool)
            chosen[sel] = True
            s_o = ref["S"][l, h]
            assert chosen[s_o > tau * (1 + EPS)].all() and not chosen[s_o < tau * (1 - EPS)].any()


# ---------------------------------------------------------------- causal tail
CAUSAL_CASES = {
    "tiny-f32": (0, dict(layers=2), {}),
    "f32-ragged-m20": (0, dict(layers=1, hq=6, hkv=2, n=777, window=20, head_dim=32), {}),
    "bf16-mfma-one-tile": (1, dict(layers=1, n=100), {}),
    "bf16-mfma-n-equals-m": (1, dict(layers=1, n=64), {}),
    "bf16-mfma-ragged": (1, dict(layers=2, n=1500), {}),
    "bf16-mfma-mask-crosses-chunk": (1, dict(layers=1, n=2048 + 30), {}),
    "bf16-mfma-mask-ends-on-tile": (1, dict(layers=1, n=2048 + 128), {}),
    "bf16-mfma-mean-task": (1, dict(layers=1, n=900), dict(agg_task=kv.KVC_AGG_MEAN)),
    "bf16-mfma-m128-gqa8": (4, dict(layers=1, n=700), {}),
    "bf16-mfma-m32-g2": (1, dict(layers=1, hq=8, hkv=4, window=32, n=500), {}),
    "bf16-mfma-noGQA": (1, dict(layers=1, hq=4, hkv=4, n=700), {}),
    "bf16-mfma-m512": (1, dict(layers=1, hq=4, hkv=2, window=512, n=600), {}),
    "bf16-mfma-m512-two-chunks": (1, dict(layers=1, hq=2, hkv=2, window=512, n=2300), {}),
    "bf16-generic-m48": (1, dict(layers=1, window=48, hq=8, hkv=4, n=400), {}),
    "bf16-varlen-batch": (3, dict(layers=1, batch=3, n_range=(200, 1400)), {}),
}


@pytest.mark.parametrize("name", list(CAUSAL_CASES))
def test_causal_tail_scores_match_oracle(name):
    cid, over, pkw = CAUSAL_CASES[name]
    _say(f"causal {name}")
    cfg = wl.get_config(cid, **over)
    w = Workload(cfg)
    dw = DeviceWorkload(w)
    p = w.params(causal_tail=1, **pkw)
    S = torch.zeros((cfg.layers, cfg.hkv, w.total), dtype=torch.float32, device="cuda")
    kv.kvc_score(p, dw.ptrs(dw.q), dw.ptrs(dw.k), w.cu, S.data_ptr(), dw.ws.data_ptr(),
                 dw.ws_bytes, stream())
    torch.cuda.synchronize()
    got = S.cpu().numpy()
    worst = 0.0
    for b in range(cfg.batch):
        lo, hi = int(w.cu[b]), int(w.cu[b + 1])
        for l in range(cfg.layers):
            ref = orc.score_layer(orc.widen(w.seq[b][l][0]), orc.widen(w.seq[b][l][1]), causal_tail=True,
                                  agg_task=pkw.get("agg_task", orc.AGG_MAX))
            np.testing.assert_allclose(got[l][:, lo:hi], ref, rtol=EPS, atol=0)
            worst = max(worst, float(np.max(np.abs(got[l][:, lo:hi] - ref) / ref)))
            # the mask matters: the last key is seen by one task token only
            plain = orc.score_layer(orc.widen(w.seq[b][l][0]), orc.widen(w.seq[b][l][1]),
                                    agg_task=pkw.get("agg_task", orc.AGG_MAX))
            if cfg.window > 1:
                assert not np.allclose(plain, ref, rtol=1e-3)
    assert worst < 1e-4, worst


def test_compress_causal_tail_end_to_end():
    cfg = wl.get_config(1, layers=3, n=2200)
    w = Workload(cfg)
    dw = DeviceWorkload(w)
    got = _run_variant(w, dw, causal_tail=1)
    ref = w.oracle(causal_tail=True)[0]
    np.testing.assert_allclose(got["S"], ref["S"], rtol=EPS)
    lens = got["lengths"][0]
    assert int(lens.sum()) == w.budgets[0]
    tau = ref["tau"]
    for l in range(cfg.layers):
        assert int((ref["I"][l] > tau * (1 + EPS)).sum()) <= int(lens[l]) <= int((ref["I"][l] >= tau * (1 - EPS)).sum())


# ------------------------------------------------------------ forced retention
@pytest.mark.parametrize("cid,over,kf,kl", [(1, dict(layers=3, n=2000), 4, 64),
                                             (3, dict(layers=2, batch=3, n_range=(300, 1500)), 2, 10),
                                             (1, dict(layers=2, n=900, hq=24, hkv=12), 3, 0)])
def test_compress_forced_retention(cid, over, kf, kl):
    _say(f"forced retention cfg={cid} first={kf} last={kl}")
    cfg = wl.get_config(cid, **over)
    w = Workload(cfg)
    dw = DeviceWorkload(w)
    got = _run_variant(w, dw, keep_first=kf, keep_last=kl)
    ref = w.oracle(keep_first=kf, keep_last=kl)
    c = cfg
    for b in range(c.batch):
        lo, hi = int(w.cu[b]), int(w.cu[b + 1])
        n = hi - lo
        forced = list(range(min(kf, n))) + list(range(max(n - kl, min(kf, n)), n))
        r = ref[b]
        S_g = got["S"][:, :, lo:hi]
        finite = np.isfinite(r["S"])
        assert np.array_equal(np.isinf(S_g), ~finite)
        np.testing.assert_allclose(S_g[finite], r["S"][finite], rtol=EPS)
        lens = got["lengths"][b]
        assert int(lens.sum()) == w.budgets[b] and int(lens.min()) >= len(forced)
        for l in range(c.layers):
            for h in range(c.hkv):
                assert got["idx"][l, h, lo:lo + len(forced)].tolist() == forced
            nl = int(lens[l])
            base = int(got["offsets"][b * c.layers + l]) * c.hkv * c.head_dim
            kblk = got["k_out"][base: base + c.hkv * nl * c.head_dim].reshape(c.hkv, nl, c.head_dim)
            for h in range(c.hkv):
                np.testing.assert_array_equal(kblk[h], w.seq[b][l][1][h, got["idx"][l, h, lo:lo + nl]])
            tau = r["tau"]
            if np.isfinite(tau):
                lo_ok = int((r["I"][l] > tau * (1 + EPS)).sum())
                hi_ok = int((r["I"][l] >= tau * (1 - EPS)).sum())
                assert lo_ok <= nl <= hi_ok
