"""The synthetic input generator: deterministic, shaped like the named
workloads, and structured (sinks and needles score high under the oracle)."""
import numpy as np
import torch

import workloads as wl
from oracle import kvc_oracle as orc


def test_configs_have_the_named_shapes():
    c0, c2, c3, c4 = (wl.get_config(i) for i in (0, 2, 3, 4))
    assert (c0.layers, c0.hq, c0.hkv, c0.head_dim, c0.n, c0.window, c0.dtype) == \
        (4, 4, 4, 64, 1024, 32, "f32")
    assert (c2.layers, c2.hq, c2.hkv, c2.head_dim, c2.n, c2.window, c2.dtype) == \
        (32, 32, 8, 128, 131072, 64, "bf16")
    assert wl.budget_for(c2, c2.n) == 419430
    assert wl.budget_for(c0, c0.n) == 1024
    lens = wl.seq_lens(c3, 0)
    assert lens.shape == (8,) and lens.min() >= 4096 and lens.max() <= 32768
    assert np.array_equal(lens, wl.seq_lens(c3, 0))
    assert (c4.layers, c4.hq, c4.hkv, c4.window, c4.group) == (80, 64, 8, 128, 8)


def test_bf16_rounding_matches_round_to_nearest_even():
    r = np.random.default_rng(0)
    x = np.concatenate([r.standard_normal(4096).astype(np.float32) * 10,
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 65280.0],
                                 dtype=np.float32)])
    ours = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(ours, ref)


def test_layers_are_deterministic_and_independent():
    cfg = wl.get_config(1, n=256, layers=3)
    a = wl.make_layer(cfg, 0, 0, 1, 256)
    b = wl.make_layer(cfg, 0, 0, 1, 256)
    c = wl.make_layer(cfg, 0, 0, 2, 256)
    d = wl.make_layer(cfg, 1, 0, 1, 256)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    assert not np.array_equal(a[1], c[1]) and not np.array_equal(a[1], d[1])
    assert a[0].dtype == np.uint16 and a[0].shape == (32, 64, 128)
    assert a[1].shape == (8, 256, 128) and a[2].shape == (8, 256, 128)


def test_sinks_and_needles_rank_high():
    cfg = wl.get_config(0)
    q, k, _ = wl.make_layer(cfg, 0, 0, 0, cfg.n, want_v=False)
    s = orc.score_layer(orc.widen(q), orc.widen(k))
    idx, _ = orc.head_rank(s)
    top = idx[:, : 4 + cfg.n_needles + 16]
    for h in range(cfg.hkv):
        assert len(set(range(4)) & set(top[h].tolist())) >= 3     # sinks
    # needle positions are shared by all heads of the layer: find them as the
    # tokens in every head's top set beyond the sinks
    common = set(top[0].tolist())
    for h in range(1, cfg.hkv):
        common &= set(top[h].tolist())
    assert len(common - set(range(4))) >= cfg.n_needles - 2


def test_query_ramp_and_key_norm_options():
    c4 = wl.get_config(4, n=64, layers=5)
    q0 = orc.widen(wl.make_layer(c4, 0, 0, 0, 64, want_v=False)[0])
    q4 = orc.widen(wl.make_layer(c4, 0, 0, 4, 64, want_v=False)[0])
    assert 0.45 < q0.std() < 0.55 and 1.9 < q4.std() < 2.1
    c3 = wl.get_config(3, n=512, n_range=None, batch=1, layers=1)
    k = orc.widen(wl.make_layer(c3, 0, 0, 0, 512, want_v=False)[1])
    norms = np.linalg.norm(k[:, 8:], axis=2) / np.sqrt(128)
    assert 0.4 < np.log(norms).std() < 0.6
