"""GPU parity of mlora_w4a8_layer_step (int8 activations, one scale per tensor; through the C ABI)
against oracle/act_quant.c.  The integer sums are exact on both sides, so the bars are those of
the bf16 path: <= 5e-3 of max|y_ref| with bf16 outputs, <= 2e-4 with fp32 outputs, and the LoRA
term on its own scale."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import TOL, TOL_F32, rel_err

pytestmark = pytest.mark.gpu


def run_a8(gpu, probs, xqs, scales, rows, M, y_dtype):
    lib, device, torch = gpu
    projs = [device.upload_problem(p) for p in probs]
    cache = {}
    dxs = []
    for xq in xqs:
        if id(xq) not in cache:
            cache[id(xq)] = torch.from_numpy(np.ascontiguousarray(xq)).cuda()
        dxs.append(cache[id(xq)])
    ys = [device.alloc_y(M, p.shape.N, y_dtype) for p in probs]
    ra = None if rows is None else torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda()
    ws = torch.zeros(max(lib.a8_workspace_bytes(projs, M), 256), dtype=torch.uint8, device="cuda")
    lib.LayerPlanA8(projs, dxs, scales, ys, ra, M, y_dtype, ws).run()
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    lib.LayerPlanA8(projs, dxs, scales, ys, ra, M, y_dtype, ws).run()      # the counters are back at zero
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    return [device.y_to_numpy(y) for y in ys]


def check_a8(gpu, probs, xqs, scales, rows, M, tag):
    y16 = run_a8(gpu, probs, xqs, scales, rows, M, 0)
    y32 = run_a8(gpu, probs, xqs, scales, rows, M, 1)
    yb32 = run_a8(gpu, probs, xqs, scales, None, M, 1)
    for i, p in enumerate(probs):
        s = p.shape
        ref = oracle.linear_a8(p.wq, p.scales, s.group, p.lora_a, p.lora_b, s.alpha, xqs[i], scales[i], rows)
        base = oracle.linear_a8(p.wq, p.scales, s.group, p.lora_a, p.lora_b, s.alpha, xqs[i], scales[i], None)
        assert rel_err(y16[i], ref) <= TOL, (tag, i, "bf16", rel_err(y16[i], ref))
        assert rel_err(y32[i], ref) <= TOL_F32, (tag, i, "fp32", rel_err(y32[i], ref))
        assert rel_err(yb32[i], base) <= TOL_F32, (tag, i, "base", rel_err(yb32[i], base))
        delta = ref - base
        if np.max(np.abs(delta)) > 0:
            assert np.max(np.abs((y32[i] - yb32[i]) - delta)) <= TOL * np.max(np.abs(delta)), (tag, i, "lora")


def shape_case(seed, K, N, G, r, n_ad, M, row_map="random"):
    shape = wl.ProjShape("t", K, N, G, r, n_ad, 2.0)
    prob = wl.make_problem(shape, 1500 + seed, 0, 0)
    xq, s = wl.make_x_int8(M, K, 1500 + seed, 0, 0)
    rng = np.random.default_rng(seed)
    rows = rng.integers(-1, n_ad, size=M).astype(np.int32)
    return [prob], [xq], [float(s)], rows


@pytest.mark.parametrize("K,N,G,r,n_ad,M", [
    (256, 64, 32, 8, 2, 1),            # one row, one tile
    (512, 200, 32, 16, 3, 8),          # N not a multiple of 64
    (2048, 2048, 32, 16, 8, 16),       # decode shape, 16 rows
    (2048, 512, 64, 16, 4, 17),
    (4096, 256, 128, 24, 3, 32),       # split K, rank not a multiple of 16
    (1152, 320, 64, 64, 5, 33),        # K / 128 not a multiple of 4
    (3072, 512, 64, 16, 16, 70),       # two row chunks, ragged
    (8192, 192, 32, 128, 2, 64),       # long K, largest rank
])
def test_a8_shapes(gpu, K, N, G, r, n_ad, M):
    probs, xqs, scales, rows = shape_case(K + N + M, K, N, G, r, n_ad, M)
    check_a8(gpu, probs, xqs, scales, rows, M, (K, N, G, r, n_ad, M))


def test_a8_extreme_codes_and_activations(gpu):
    """Every code -8 or +7 against activations of +-127 only: the largest group sums the int32
    accumulators and the bias trick have to hold (2 k-steps x 32 inputs x 8 x 16 x 127)."""
    probs, xqs, scales, rows = shape_case(99, 1024, 128, 64, 16, 2, 24)
    p = probs[0]
    rng = np.random.default_rng(1)
    p.wq[:] = np.where(rng.random(p.wq.shape) < 0.5, 0x88, 0x77).astype(np.uint8)
    p.wq[0] = 0x88
    p.wq[1] = 0x77
    xqs[0][:] = np.where(rng.random(xqs[0].shape) < 0.5, -127, 127).astype(np.int8)
    xqs[0][0] = 127
    xqs[0][1] = -127
    check_a8(gpu, probs, xqs, scales, rows, 24, "extreme")


def test_a8_full_layer_c2_and_c4_decode_rows(gpu):
    """All seven projections of a 1B-like layer in one call, at 8 rows (c2) and 32 rows (c4 decode)."""
    for key in ("c2", "c4_decode"):
        w = wl.WORKLOADS[key]
        probs = [wl.make_problem(s, w.cfg_id, 0, i) for i, s in enumerate(w.projs)]
        slots = {}
        xqs, scales = [], []
        for i, s in enumerate(w.projs):
            if s.K not in slots:
                slots[s.K] = wl.make_x_int8(w.M, s.K, w.cfg_id, 0, len(slots))
            xqs.append(slots[s.K][0])
            scales.append(float(slots[s.K][1]))
        rows = wl.make_rows(w.row_map, w.M, w.projs[0].n_adapters, w.cfg_id)
        check_a8(gpu, probs, xqs, scales, rows, w.M, key)


def test_a8_c3_and_c5_shapes(gpu):
    for key in ("c3", "c5_up"):
        w = wl.WORKLOADS[key]
        probs = [wl.make_problem(s, w.cfg_id, 0, i) for i, s in enumerate(w.projs)]
        xqs, scales = [], []
        for i, s in enumerate(w.projs):
            xq, sc = wl.make_x_int8(w.M, s.K, w.cfg_id, 0, i)
            xqs.append(xq)
            scales.append(float(sc))
        rows = wl.make_rows(w.row_map, w.M, w.projs[0].n_adapters, w.cfg_id)
        check_a8(gpu, probs, xqs, scales, rows, w.M, key)


def test_a8_rejects_bad_scales(gpu):
    lib, device, torch = gpu
    probs, xqs, scales, rows = shape_case(5, 256, 64, 32, 8, 2, 4)
    projs = [device.upload_problem(probs[0])]
    x = torch.from_numpy(xqs[0]).cuda()
    y = device.alloc_y(4, 64, 0)
    ws = torch.zeros(max(lib.a8_workspace_bytes(projs, 4), 256), dtype=torch.uint8, device="cuda")
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(lib.MloraError):
            lib.LayerPlanA8(projs, [x], [bad], [y], None, 4, 0, ws).run()
