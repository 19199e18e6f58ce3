"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

import paper_2509_05165_amd as kv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000          # a non-null "device pointer" that is never dereferenced on error paths


def declared_functions():
    text = open(os.path.join(ROOT, "include", "kvc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"kvc_compress", "kvc_score", "kvc_head_rank", "kvc_composite", "kvc_global_select",
            "kvc_gather", "kvc_workspace_size", "kvc_budget"} <= set(names)
    lib = ctypes.CDLL(kv.lib_path())
    for n in names:
        assert hasattr(lib, n), f"{n} declared in kvc.h but not exported"


def test_version_status_strings_and_budget():
    assert kv.kvc_version() >= 100
    assert kv.kvc_status_string(0) == "KVC_OK"
    assert kv.kvc_status_string(3) == "KVC_ERR_WORKSPACE"
    assert kv.kvc_budget(10, 32, 131072) == 419430          # floor(0.1 * 32 * 131072)
    assert kv.kvc_budget(25, 4, 1024) == 1024
    assert kv.kvc_budget(20, 32, 4097) == (20 * 32 * 4097) // 100
    assert kv.kvc_budget(101, 1, 1) == -1


def P(**kw):
    base = dict(batch=1, layers=2, hq=8, hkv=4, head_dim=128, window=64, dtype=kv.KVC_BF16)
    base.update(kw)
    return kv.KvcParams(**base)


def expect(status, fn, *a, **k):
    with pytest.raises(kv.KvcError) as e:
        fn(*a, **k)
    assert e.value.status == status, str(e.value)
    assert kv.kvc_last_error() != ""


def test_workspace_size_grows_with_problem():
    a = kv.kvc_workspace_size(P(), 1000, 1000)
    b = kv.kvc_workspace_size(P(), 4000, 4000)
    c = kv.kvc_workspace_size(P(layers=4), 4000, 4000)
    assert 0 < a < b < c
    assert a % 256 == 0
    expect(1, kv.kvc_workspace_size, P(), 10, 20)           # max_seqlen > total


@pytest.mark.parametrize("bad", [
    dict(hq=6, hkv=4), dict(window=0), dict(layers=0), dict(dtype=7), dict(agg_task=3),
    dict(add_head_mean=2), dict(softmax_scale=-1.0), dict(softmax_scale=float("nan"))])
def test_invalid_params(bad):
    expect(1, kv.kvc_workspace_size, P(**bad), 100, 100)
    expect(1, kv.kvc_score, P(**bad), [FAKE] * 2, [FAKE] * 2, [0, 100], FAKE, FAKE, 1 << 30)


@pytest.mark.parametrize("bad", [
    dict(head_dim=12), dict(head_dim=512), dict(batch=257), dict(layers=129), dict(window=5000)])
def test_unsupported_params(bad):
    expect(2, kv.kvc_workspace_size, P(**bad), 100, 100)


def test_sequence_table_checks():
    p = P(batch=2)
    expect(1, kv.kvc_composite, p, FAKE, [1, 5, 9], FAKE)            # cu[0] != 0
    expect(1, kv.kvc_composite, p, FAKE, [0, 9, 5], FAKE)            # decreasing
    expect(2, kv.kvc_composite, p, FAKE, [0, 5, 1 << 31], FAKE)      # too many tokens
    expect(2, kv.kvc_composite, p, FAKE, [0, 5, 5 + (1 << 29)], FAKE)  # one sequence of 2^29 tokens
    expect(1, kv.kvc_composite, p, 0, [0, 5, 9], FAKE)               # null S_sorted
    expect(1, kv.kvc_composite, p, FAKE, [0, 5, 9], 0)               # null I


def test_null_pointers_and_tables():
    p = P()
    cu = [0, 100]
    big = 1 << 30
    expect(1, kv.kvc_score, p, [FAKE, 0], [FAKE] * 2, cu, FAKE, FAKE, big)        # q[1] null
    expect(1, kv.kvc_score, p, [FAKE] * 2, None, cu, FAKE, FAKE, big)             # k table null
    expect(1, kv.kvc_score, p, [FAKE] * 2, [FAKE] * 2, cu, 0, FAKE, big)          # S null
    expect(1, kv.kvc_head_rank, p, FAKE, cu, 0, FAKE, FAKE, big)
    expect(1, kv.kvc_global_select, p, FAKE, cu, [10], FAKE, 0, FAKE, FAKE, big)  # lengths null
    expect(1, kv.kvc_gather, p, [FAKE] * 2, [FAKE] * 2, FAKE, FAKE, FAKE, cu, 10, FAKE, 0)  # v w/o v_out
    expect(1, kv.kvc_gather, p, [FAKE] * 2, None, FAKE, FAKE, FAKE, cu, 10, 0, 0)  # k_out null
    expect(1, kv.kvc_compress, p, [FAKE] * 2, [FAKE] * 2, [FAKE] * 2, cu, [10], FAKE, 0,
           FAKE, FAKE, FAKE, big)                                                 # v w/o v_out
    expect(1, kv.kvc_compress, p, [FAKE] * 2, [FAKE] * 2, [FAKE] * 2, cu, [10], FAKE, FAKE,
           0, FAKE, FAKE, big)                                                    # lengths null


def test_budget_range():
    p = P()
    cu = [0, 100]
    big = 1 << 30
    expect(1, kv.kvc_global_select, p, FAKE, cu, [201], FAKE, FAKE, FAKE, FAKE, big)  # > layers*N
    expect(1, kv.kvc_global_select, p, FAKE, cu, [-1], FAKE, FAKE, FAKE, FAKE, big)
    expect(1, kv.kvc_gather, p, [FAKE] * 2, [FAKE] * 2, FAKE, FAKE, FAKE, cu, 201, FAKE, FAKE)
    expect(1, kv.kvc_compress, p, [FAKE] * 2, [FAKE] * 2, [FAKE] * 2, cu, [201], FAKE, FAKE,
           FAKE, FAKE, FAKE, big)


def test_workspace_checks():
    p = P()
    cu = [0, 100]
    need = kv.kvc_workspace_size(p, 100, 100)
    args = (p, [FAKE] * 2, [FAKE] * 2, [FAKE] * 2, cu, [10], FAKE, FAKE, FAKE, FAKE)
    expect(3, kv.kvc_compress, *args, FAKE, need - 1)         # too small
    expect(3, kv.kvc_compress, *args, 0, need)                # missing
    expect(3, kv.kvc_compress, *args, FAKE + 8, need)         # misaligned
    expect(3, kv.kvc_score, p, [FAKE] * 2, [FAKE] * 2, cu, FAKE, FAKE, 16)
    expect(3, kv.kvc_head_rank, p, FAKE, cu, FAKE, FAKE, FAKE, 16)


def test_empty_problem_is_a_no_op_without_gpu():
    # zero tokens: nothing to enqueue for the per-token stages, so they return OK on any host
    p = P()
    kv.kvc_score(p, [FAKE] * 2, [FAKE] * 2, [0, 0], FAKE, FAKE, 1 << 20)
    kv.kvc_head_rank(p, FAKE, [0, 0], FAKE, FAKE, FAKE, 1 << 20)
    kv.kvc_composite(p, FAKE, [0, 0], FAKE)
    kv.kvc_gather(p, [FAKE] * 2, [FAKE] * 2, FAKE, FAKE, FAKE, [0, 0], 0, FAKE, FAKE)


def test_variant_parameter_checks():
    expect(1, kv.kvc_workspace_size, P(value_norm=2), 100, 100)
    expect(1, kv.kvc_workspace_size, P(order=2), 100, 100)
    expect(1, kv.kvc_workspace_size, P(min_per_layer=-1), 100, 100)
    expect(1, kv.kvc_workspace_size, P(unstructured=3), 100, 100)
    expect(1, kv.kvc_workspace_size, P(causal_tail=2), 100, 100)
    # the variants never need less workspace than the plain pass
    base = kv.kvc_workspace_size(P(), 50000, 50000)
    assert kv.kvc_workspace_size(P(value_norm=1), 50000, 50000) >= base
    assert kv.kvc_workspace_size(P(order=kv.KVC_ORDER_POSITION), 50000, 50000) >= base


def test_variant_argument_checks_run_before_any_gpu_call():
    cu = [0, 100]
    # value norms need the value pointers
    expect(1, kv.kvc_score, P(value_norm=1), [FAKE] * 2, [FAKE] * 2, cu, FAKE, FAKE, 1 << 30)
    # a budget below layers * floor cannot be met
    expect(1, kv.kvc_global_select, P(min_per_layer=10), FAKE, cu, [19], 0, FAKE, FAKE, FAKE, 1 << 30)
    # unstructured: the budget counts (head, token) entries, up to layers*hkv*N
    expect(1, kv.kvc_global_select, P(unstructured=1), FAKE, cu, [2 * 4 * 100 + 1], 0, FAKE, FAKE, FAKE, 1 << 30)
    # the causal tail needs at least as many cached tokens as task tokens
    expect(1, kv.kvc_score, P(causal_tail=1), [FAKE] * 2, [FAKE] * 2, [0, 63], FAKE, FAKE, 1 << 30)
    # position order needs workspace in the gather stage
    expect(3, kv.kvc_gather, P(order=kv.KVC_ORDER_POSITION), [FAKE] * 2, [FAKE] * 2, FAKE, FAKE, FAKE,
           cu, 5, FAKE, FAKE, 0)


def test_static_select_rejects_what_its_buffer_cannot_hold():
    # 64 sequences x 128 rows of 2^24 tokens need far more ticket lines than the
    # built-in buffer holds: refused on the host, nothing enqueued
    import numpy as np
    lyr, bt = 128, 64
    n = (1 << 30) // bt - 1
    p = kv.KvcParams(bt, lyr, 8, 8, 128, 64, kv.KVC_BF16)
    cu = [i * n for i in range(bt + 1)]
    expect(2, kv.kvc_global_select_static, p, FAKE, cu, [0] * bt, 0, FAKE, FAKE)
    # and the argument checks of kvc_global_select apply unchanged
    expect(1, kv.kvc_global_select_static, P(), FAKE, [0, 100], [10 ** 9], 0, FAKE, FAKE)
    expect(1, kv.kvc_global_select_static, P(), FAKE, [0, 100], [10], 0, 0, FAKE)


def test_bench_traffic_file_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    """bench.py hands out counter-derived HBM bytes only while the kernel sources still
    have the digest the figures were recorded with."""
    import importlib.util
    import json
    spec = importlib.util.spec_from_file_location("kvc_bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    shape = {"hq": 32, "hkv": 8, "head_dim": 128, "window": 64, "tokens": 131072}
    good = {"commit": "abc", "kernel_source_digest": bench.kernel_source_digest(), "layer_shape": shape,
            "fetch_scale": 2.0, "write_scale": 1.0,
            "kernels": {"score_mfma<stats>": {"bytes_per_layer": 274.3e6}}}
    f = tmp_path / "t.json"
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    assert bench.load_traffic("score_mfma<stats>", shape)[0] is None          # no file
    f.write_text(json.dumps(good))
    per_layer, note = bench.load_traffic("score_mfma<stats>", shape)
    assert per_layer == 274.3e6 and "abc" in note
    assert bench.load_traffic("score_mfma<emit>", shape)[0] is None           # kernel not recorded
    assert bench.load_traffic("score_mfma<stats>", dict(shape, tokens=1))[0] is None
    f.write_text(json.dumps(dict(good, kernel_source_digest="0" * 16)))
    per_layer, note = bench.load_traffic("score_mfma<stats>", shape)
    assert per_layer is None and "stale" in note
