"""mlora_w4_layer_step_static (the entry point that allocates nothing) against
mlora_w4_layer_step: same kernels, so the outputs must be bit-identical; two calls in a row on
the shared built-in scratch, the second with a smaller input, then a larger one again."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import TOL_F32, rel_err

pytestmark = pytest.mark.gpu


def both_ways(gpu, probs, projs, xs, rows, M, y_dtype):
    lib, device, torch = gpu
    dxs = [device.to_device(np.ascontiguousarray(x[:M])) for x in xs]
    ra = torch.from_numpy(np.ascontiguousarray(rows[:M], np.int32)).cuda()
    ys_a = [device.alloc_y(M, p.shape.N, y_dtype) for p in probs]
    ys_b = [device.alloc_y(M, p.shape.N, y_dtype) for p in probs]
    for y in ys_a + ys_b:
        y.fill_(-3)
    ws = device.alloc_workspace(projs, M)
    lib.layer_step(projs, dxs, ys_a, ra, M, y_dtype, ws)
    lib.layer_step_static(projs, dxs, ys_b, ra, M, y_dtype)
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    for p, ya, yb in zip(probs, ys_a, ys_b):
        assert torch.equal(ya, yb), p.shape.name
    return [device.y_to_numpy(y) for y in ys_b]


def test_static_scratch_entry_point_matches_the_workspace_one(gpu):
    lib, device, torch = gpu
    shapes = [wl.ProjShape("a", 4096, 200, 32, 16, 4, 2.0), wl.ProjShape("b", 512, 328, 64, 24, 4, 2.0),
              wl.ProjShape("c", 2304, 96, 128, 8, 4, 2.0)]
    probs = [wl.make_problem(s, 79, 0, i) for i, s in enumerate(shapes)]
    projs = [device.upload_problem(p) for p in probs]
    rng = np.random.default_rng(79)
    xs = [wl.f32_to_bf16_bits(rng.standard_normal((100, s.K)).astype(np.float32)) for s in shapes]
    rows = rng.integers(-1, 4, size=100).astype(np.int32)
    # a wide call, then smaller ones of other geometries on the same scratch, then a larger one again
    for M, y_dtype in [(100, lib.Y_FP32), (24, lib.Y_FP32), (7, lib.Y_BF16), (70, lib.Y_BF16), (1, lib.Y_FP32)]:
        got = both_ways(gpu, probs, projs, xs, rows, M, y_dtype)
        if y_dtype == lib.Y_FP32:
            for p, x, y in zip(probs, xs, got):
                ref = oracle.linear(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha,
                                    np.ascontiguousarray(x[:M]), np.ascontiguousarray(rows[:M]))
                assert rel_err(y, ref) <= TOL_F32, (M, p.shape.name)


def test_static_scratch_rejects_what_does_not_fit(gpu):
    lib, device, torch = gpu
    # K = 16384 at 4096 rows: the split-K partial tiles alone are far beyond the built-in scratch
    shape = wl.ProjShape("big", 16384, 8192, 32, 16, 2, 1.0)
    fake = lib.Proj(shape.K, shape.N, shape.group, torch.zeros(16, dtype=torch.uint8, device="cuda"),
                    torch.zeros((2, 16, 16), dtype=torch.int16, device="cuda"),
                    torch.zeros((2, 16, 16), dtype=torch.int16, device="cuda"), 1.0, n_adapters=2, rank=16)
    x = torch.zeros(16, dtype=torch.int16, device="cuda")
    y = torch.zeros(16, dtype=torch.int16, device="cuda")
    ra = torch.zeros(4096, dtype=torch.int32, device="cuda")
    with pytest.raises(lib.MloraError) as e:
        lib.layer_step_static([fake], [x], [y], ra, 4096)       # refused on the host: nothing is launched
    assert e.value.status == -4
