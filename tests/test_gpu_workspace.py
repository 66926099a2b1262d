"""The workspace contract on the GPU: one workspace sized for the largest call serves calls of
different geometry one after another; a wait that runs out is reported and poisons the output;
rows whose adapter index is out of range are computed without adapter; calls with more
projections than one launch holds."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import TOL_F32, random_problem, rel_err

pytestmark = pytest.mark.gpu


def oracle_y(p, x, rows):
    return oracle.linear(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha, x, rows)


def test_one_workspace_serves_calls_of_different_geometry(gpu):
    """The seven projections of a decoder layer in dependency order (q, k, v | o | gate, up |
    down) as separate calls on ONE workspace sized for the largest need, then a 64-row call and
    a 24-row call on the same workspace: the counter lines of a later call lie where an earlier
    call of another geometry kept nothing but zeros."""
    lib, device, torch = gpu
    w = wl.WORKLOADS["c2"]
    probs, xs, rows = wl.make_layer(w, layer=5)
    projs = [device.upload_problem(p) for p in probs]
    rng = np.random.default_rng(2)
    cases = [(8, i) for i in (0, 1, 2, 3, 4, 5, 6)] + [(64, 6), (24, 0), (8, 6), (130, 4), (8, 3)]
    n_ws = max(lib.workspace_bytes([projs[i]], M) for M, i in cases)
    ws = torch.empty(n_ws, dtype=torch.uint8, device="cuda")
    lib.workspace_init(ws)
    for M, i in cases:
        p = probs[i]
        x = wl.f32_to_bf16_bits(rng.standard_normal((M, p.shape.K)).astype(np.float32))
        ra = rng.integers(-1, p.shape.n_adapters, size=M).astype(np.int32)
        y = device.alloc_y(M, p.shape.N, lib.Y_FP32)
        lib.linear(projs[i], device.to_device(x), torch.from_numpy(ra).cuda(), M, y, lib.Y_FP32, ws)
        torch.cuda.synchronize()
        assert lib.workspace_status(ws) == 0
        assert rel_err(device.y_to_numpy(y), oracle_y(p, x, ra)) <= TOL_F32, (M, p.shape.name)


def test_a_wait_that_runs_out_is_reported_and_poisons_the_output(gpu):
    """With the spin limit forced to 0 every wait gives up at once (all kernels still run to
    their end): the status word is set and the waiting blocks store NaN.  After
    mlora_w4_workspace_init the same workspace works again."""
    lib, device, torch = gpu
    for K, N, M in [(4096, 128, 8), (4096, 128, 24), (1024, 256, 70)]:
        prob = random_problem(K + M, K, N, 32, 16, 4)
        proj = device.upload_problem(prob)
        rng = np.random.default_rng(M)
        x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
        ra = rng.integers(0, 4, size=M).astype(np.int32)
        dx, dra = device.to_device(x), torch.from_numpy(ra).cuda()
        y = device.alloc_y(M, N, lib.Y_FP32)
        ws = device.alloc_workspace([proj], M)
        old = lib.debug_spin_limit(0)
        try:
            lib.linear(proj, dx, dra, M, y, lib.Y_FP32, ws)
            torch.cuda.synchronize()
        finally:
            lib.debug_spin_limit(old)
        assert lib.workspace_status(ws) != 0
        assert bool(torch.isnan(y).all().item()), "every output waits for the shrink step here"
        lib.workspace_init(ws)
        lib.linear(proj, dx, dra, M, y, lib.Y_FP32, ws)
        torch.cuda.synchronize()
        assert lib.workspace_status(ws) == 0
        assert rel_err(device.y_to_numpy(y), oracle_y(prob, x, ra)) <= TOL_F32


@pytest.mark.parametrize("M", [6, 30, 80])
def test_out_of_range_adapter_rows_are_computed_without_adapter(gpu, M):
    lib, device, torch = gpu
    prob = random_problem(50 + M, 512, 200, 64, 16, 5)
    rng = np.random.default_rng(M)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, 512)).astype(np.float32))
    ra = rng.integers(0, 5, size=M).astype(np.int32)
    ra[1], ra[M // 2], ra[M - 1] = 5, -7, 1 << 20        # n_adapters itself, negative, far beyond
    proj = device.upload_problem(prob)
    y = device.alloc_y(M, 200, lib.Y_FP32)
    ws = device.alloc_workspace([proj], M)
    lib.linear(proj, device.to_device(x), torch.from_numpy(ra).cuda(), M, y, lib.Y_FP32, ws)
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    as_base = np.where((ra < 0) | (ra >= 5), -1, ra).astype(np.int32)
    ref = oracle_y(prob, x, as_base)
    got = device.y_to_numpy(y)
    assert rel_err(got, ref) <= TOL_F32
    bad = [1, M // 2, M - 1]
    assert rel_err(got[bad], oracle_y(prob, x[bad], None)) <= TOL_F32


@pytest.mark.parametrize("M", [4, 20])
def test_more_projections_than_one_launch_holds(gpu, M):
    """150 small projections: a launch of 128 (eight groups of 16) and one of 22."""
    lib, device, torch = gpu
    rng = np.random.default_rng(150 + M)
    shapes = [wl.ProjShape(f"p{i}", [128, 256, 2176][i % 3], [64, 80, 130][(i // 3) % 3], 32, 8, 3, 1.0)
              for i in range(150)]
    base = [wl.make_problem(s, 78, 0, i) for i, s in enumerate(shapes[:9])]
    probs = [base[i % 9] for i in range(150)]
    uploaded = [device.upload_problem(p) for p in base]
    projs = [uploaded[i % 9] for i in range(150)]
    xs_by_k = {K: wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)) for K in (128, 256, 2176)}
    dx_by_k = {K: device.to_device(v) for K, v in xs_by_k.items()}
    rows = rng.integers(-1, 3, size=M).astype(np.int32)
    ys = [device.alloc_y(M, p.shape.N, lib.Y_FP32) for p in probs]
    ws = device.alloc_workspace(projs, M)
    lib.layer_step(projs, [dx_by_k[p.shape.K] for p in probs], ys, torch.from_numpy(rows).cuda(), M, lib.Y_FP32, ws)
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    refs = [oracle_y(p, xs_by_k[p.shape.K], rows) for p in base]
    for i, y in enumerate(ys):
        assert rel_err(device.y_to_numpy(y), refs[i % 9]) <= TOL_F32, i
