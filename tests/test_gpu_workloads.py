"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times: all projections of the workload (for the 16-layer stack: all 112 of them) in ONE
mlora_w4_layer_step call, every layer compared with the oracle on all N output columns.

Per projection three things are checked against the fp64 oracle: the bf16 output (<= 5e-3 of
max|y_ref|), the fp32 output (<= 2e-4), and the LoRA term on its own scale (y - y_base against
the oracle's y - y_base, <= 5e-3 of the largest delta), so that a wrong adapter, a dropped
alpha or a missing row cannot hide below the size of the base product.
"""
import functools

import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import TOL, TOL_F32, assert_workspace_clean, rel_err

pytestmark = pytest.mark.gpu


@functools.lru_cache(maxsize=None)
def problems_of(key, layer):
    """Frozen tensors of one layer of a workload (c4_decode and c4_prefill share theirs: same seeds)."""
    w = wl.WORKLOADS[key]
    return tuple(wl.make_problem(s, w.cfg_id, layer, i) for i, s in enumerate(w.projs))


_device_projs = {}


def device_projs(gpu, key, layer):
    lib, device, torch = gpu
    w = wl.WORKLOADS[key]
    ck = (w.cfg_id, tuple(w.projs), layer)
    if ck not in _device_projs:
        _device_projs[ck] = [device.upload_problem(p) for p in problems_of(key, layer)]
    return _device_projs[ck]


def run_stack(gpu, key, layers, rows, y_dtype, with_rows=True):
    """One layer_step call over all projections of `layers`; returns per layer the list of outputs."""
    lib, device, torch = gpu
    w = wl.WORKLOADS[key]
    projs, dxs, shapes = [], [], []
    for layer in layers:
        _, xs, _ = wl.make_layer_inputs(w, layer)
        cache = {}
        for x in xs:
            if id(x) not in cache:
                cache[id(x)] = device.to_device(x)
            dxs.append(cache[id(x)])
        projs += device_projs(gpu, key, layer)
        shapes += [p.shape for p in problems_of(key, layer)]
    ra = torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda() if with_rows else None
    ys = [device.alloc_y(w.M, s.N, y_dtype) for s in shapes]
    ws = device.alloc_workspace(projs, w.M)
    lib.layer_step(projs, dxs, ys, ra, w.M, y_dtype, ws)
    torch.cuda.synchronize()
    assert_workspace_clean(gpu, ws, shapes, w.M)
    out = [device.y_to_numpy(y) for y in ys]
    n = len(w.projs)
    return [out[i * n:(i + 1) * n] for i in range(len(layers))]


def check_stack(gpu, key, layers, rows=None, row_sample=None):
    """Compare every projection of every layer with the oracle on all N columns (rows: all of
    them, or the given sample)."""
    w = wl.WORKLOADS[key]
    if rows is None:
        rows = wl.make_rows(w.row_map, w.M, w.projs[0].n_adapters, w.cfg_id)
    msel = np.arange(w.M) if row_sample is None else np.asarray(row_sample)
    y16 = run_stack(gpu, key, layers, rows, 0)
    y32 = run_stack(gpu, key, layers, rows, 1)
    yb32 = run_stack(gpu, key, layers, rows, 1, with_rows=False)
    worst = [0.0, 0.0, 0.0]
    for li, layer in enumerate(layers):
        _, xs, _ = wl.make_layer_inputs(w, layer)
        for pi, (p, x) in enumerate(zip(problems_of(key, layer), xs)):
            args = (p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha, np.ascontiguousarray(x[msel]))
            ref = oracle.linear(*args, np.ascontiguousarray(rows[msel]))
            base = oracle.linear(*args, None)
            e16 = rel_err(y16[li][pi][msel], ref)
            e32 = rel_err(y32[li][pi][msel], ref)
            eb = rel_err(yb32[li][pi][msel], base)
            delta = ref - base
            ed = float(np.max(np.abs((y32[li][pi][msel] - yb32[li][pi][msel]) - delta)) / np.max(np.abs(delta)))
            tag = f"{key} layer {layer} {p.shape.name}"
            assert e16 <= TOL and e32 <= TOL_F32 and eb <= TOL_F32 and ed <= TOL, (tag, e16, e32, eb, ed)
            worst = [max(a, b) for a, b in zip(worst, (e16, e32, ed))]
    print(f"{key}: {len(layers)} layer(s), worst bf16 {worst[0]:.2e}, fp32 {worst[1]:.2e}, "
          f"LoRA term {worst[2]:.2e}", flush=True)


def test_config2_layer_step_all_projections(gpu):
    check_stack(gpu, "c2", [0])


def test_config4_decode_all_16_layers_in_one_call(gpu):
    """112 projections, M = 32, one call (one launch): every layer, every row, every column."""
    check_stack(gpu, "c4_decode", list(range(16)))


def prefill_row_sample():
    rng = np.random.default_rng(11)
    inner = rng.choice(np.arange(1, 511), size=38, replace=False)
    # first and last row of the call, both sides of every 64-row chunk boundary near the middle
    return np.sort(np.unique(np.concatenate([[0, 511, 63, 64, 255, 256], inner])))


def test_config4_prefill_all_16_layers_in_one_call(gpu):
    """M = 512 rows of adapter 0 (the paper's own case: one LoRA per execution), all layers in
    one call; oracle on all N columns of 44 rows that include the first and the last."""
    check_stack(gpu, "c4_prefill", list(range(16)), row_sample=prefill_row_sample())


def test_config4_prefill_with_a_nonzero_adapter(gpu):
    w = wl.WORKLOADS["c4_prefill"]
    check_stack(gpu, "c4_prefill", [0, 7], rows=np.full(w.M, 5, np.int32), row_sample=prefill_row_sample())


@pytest.mark.parametrize("key", ["c3", "c3_interleaved"])
def test_config3_tree_rows(gpu, key):
    """8 streams x 16 draft-tree tokens, stream-major and node-major row order."""
    check_stack(gpu, key, [0])


@pytest.mark.parametrize("key", ["c5_up", "c5_down"])
def test_config5_zipf_all_columns(gpu, key):
    check_stack(gpu, key, [0])


def test_config4_decode_layer_by_layer_matches_the_single_call(gpu):
    """The same stack as sixteen calls of seven projections gives bit-identical outputs."""
    rows = wl.make_rows("block:4", 32, 8, 4)
    one = run_stack(gpu, "c4_decode", [2, 3], rows, 0)
    for i, layer in enumerate([2, 3]):
        sep = run_stack(gpu, "c4_decode", [layer], rows, 0)[0]
        assert all(np.array_equal(a, b) for a, b in zip(one[i], sep))
