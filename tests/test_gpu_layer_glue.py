"""GPU parity of mlora_w4_layer_step_fused and mlora_rms_scale (through the C ABI) against
oracle/layer_glue.py, at row counts that reach every kind of block the library has (tile blocks
with the short and the general way out, blocks of four column tiles), and a whole decoder layer
built from those calls and the tree attention."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import TOL, TOL_F32, rel_err
from oracle import layer_glue as glue
from workloads.generate import bf16_bits_to_f32, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def dev_f32(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()


def run_fused(gpu, probs, xs, rows, M, y_dtype, specs):
    """specs[i]: dict(row_scale=f32 [M] | None, pair='none'|'rope'|'swiglu', cos, sin, residual=bits | None)."""
    lib, device, torch = gpu
    projs = [device.upload_problem(p) for p in probs]
    dxs = [device.to_device(x) for x in xs]
    epis, ys = [], []
    for p, sp in zip(probs, specs):
        pair = {"none": lib.PAIR_NONE, "rope": lib.PAIR_ROPE, "swiglu": lib.PAIR_SWIGLU}[sp.get("pair", "none")]
        epis.append(lib.Epilogue(
            None if sp.get("row_scale") is None else dev_f32(torch, sp["row_scale"]), pair,
            None if sp.get("cos") is None else dev_f32(torch, sp["cos"]),
            None if sp.get("sin") is None else dev_f32(torch, sp["sin"]),
            None if sp.get("residual") is None else device.to_device(sp["residual"])))
        n_out = p.shape.N // 2 if pair == lib.PAIR_SWIGLU else p.shape.N
        ys.append(device.alloc_y(M, n_out, y_dtype))
    ra = None if rows is None else torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda()
    ws = device.alloc_workspace(projs, M)
    lib.LayerPlanFused(projs, epis, dxs, ys, ra, M, y_dtype, ws).run()
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    return [device.y_to_numpy(y) for y in ys]


def reference(probs, xs, rows, specs):
    out = []
    for p, x, sp in zip(probs, xs, specs):
        s = p.shape
        out.append(glue.fused_linear(p.wq, p.scales, s.group, p.lora_a, p.lora_b, s.alpha, x, rows,
                                     sp.get("row_scale"), sp.get("pair", "none"), sp.get("cos"), sp.get("sin"),
                                     sp.get("residual")))
    return out


def make_specs(rng, probs, M, kinds):
    specs = []
    for p, kind in zip(probs, kinds):
        sp = {}
        n_out = p.shape.N // 2 if kind == "swiglu" else p.shape.N
        if "scale" in kind or kind in ("rope", "swiglu", "all"):
            sp["row_scale"] = rng.uniform(0.3, 3.0, M).astype(np.float32)
        if kind in ("rope", "all"):
            ang = glue.rope_angles(rng.integers(0, 4096, M))
            sp.update(pair="rope", cos=np.cos(ang).astype(np.float32), sin=np.sin(ang).astype(np.float32))
        if kind == "swiglu":
            sp["pair"] = "swiglu"
        if kind in ("residual", "all", "swiglu"):
            sp["residual"] = f32_to_bf16_bits(rng.standard_normal((M, n_out)).astype(np.float32))
        specs.append(sp)
    return specs


@pytest.mark.parametrize("M", [1, 8, 16, 24, 32, 48, 70])
def test_fused_outputs_match_oracle(gpu, M):
    """Three projections in one call: q with scale + RoPE + residual, gate/up fused with SwiGLU +
    residual, o with a residual only; plus one with no operation at all (the plain path inside a
    fused call)."""
    rng = np.random.default_rng(M)
    K = 512
    pq = wl.make_problem(wl.ProjShape("q", K, 256, 32, 16, 3, 2.0), 2100 + M, 0, 0)
    pg = wl.make_problem(wl.ProjShape("gate", K, 192, 32, 8, 3, 2.0), 2100 + M, 0, 1)
    pu = wl.make_problem(wl.ProjShape("up", K, 192, 32, 8, 3, 2.0), 2100 + M, 0, 2)
    po = wl.make_problem(wl.ProjShape("o", K, 200, 32, 16, 3, 2.0), 2100 + M, 0, 3)
    pn = wl.make_problem(wl.ProjShape("n", K, 64, 32, 16, 3, 2.0), 2100 + M, 0, 4)
    probs = [pq, wl.fuse_gate_up(pg, pu), po, pn]
    x = wl.make_x(M, K, 2100 + M, 0, 0)
    xs = [x, x, x, x]
    rows = rng.integers(-1, 3, M).astype(np.int32)
    specs = make_specs(rng, probs, M, ["all", "swiglu", "residual", "none"])
    ref = reference(probs, xs, rows, specs)
    for y_dtype, tol in ((0, TOL), (1, TOL_F32)):
        got = run_fused(gpu, probs, xs, rows, M, y_dtype, specs)
        for i in range(len(probs)):
            assert rel_err(got[i], ref[i]) <= tol, (M, i, y_dtype, rel_err(got[i], ref[i]))


@pytest.mark.parametrize("M,K,rank", [(8, 4096, 32), (20, 2048, 64), (16, 16384, 16)])
def test_fused_outputs_on_the_general_way_out(gpu, M, K, rank):
    """Ranks above 16 and many split-K units take the tile blocks' general output code."""
    rng = np.random.default_rng(K + M)
    pq = wl.make_problem(wl.ProjShape("q", K, 128, 64, rank, 2, 2.0), 2200 + M, 0, 0)
    pg = wl.make_problem(wl.ProjShape("gate", K, 64, 64, rank, 2, 2.0), 2200 + M, 0, 1)
    pu = wl.make_problem(wl.ProjShape("up", K, 64, 64, rank, 2, 2.0), 2200 + M, 0, 2)
    probs = [pq, wl.fuse_gate_up(pg, pu)]
    x = wl.make_x(M, K, 2200 + M, 0, 0)
    rows = rng.integers(-1, 2, M).astype(np.int32)
    specs = make_specs(rng, probs, M, ["all", "swiglu"])
    ref = reference(probs, [x, x], rows, specs)
    got = run_fused(gpu, probs, [x, x], rows, M, 1, specs)
    for i in range(2):
        assert rel_err(got[i], ref[i]) <= TOL_F32, (i, rel_err(got[i], ref[i]))


def test_fused_outputs_in_a_long_launch_of_17_to_32_rows(gpu):
    """Ten wide projections at 24 rows: 320 blocks of four column tiles, the family a launch of
    300 and more such blocks runs at 17 to 32 rows."""
    lib, device, torch = gpu
    rng = np.random.default_rng(77)
    M, K = 24, 256
    probs = [wl.make_problem(wl.ProjShape("p%d" % i, K, 8192, 32, 16, 2, 2.0), 2500, 0, i) for i in range(10)]
    info = lib.layer_step_plan([device.upload_problem(probs[0])] * 10, M)
    assert info["wide"] and info["rows_per_chunk"] == 32
    x = wl.make_x(M, K, 2500, 0, 0)
    rows = rng.integers(-1, 2, M).astype(np.int32)
    kinds = ["all", "swiglu", "residual", "none", "rope", "swiglu", "all", "none", "residual", "rope"]
    specs = make_specs(rng, probs, M, kinds)
    ref = reference(probs, [x] * 10, rows, specs)
    got = run_fused(gpu, probs, [x] * 10, rows, M, 1, specs)
    for i in range(10):
        assert rel_err(got[i], ref[i]) <= TOL_F32, (i, rel_err(got[i], ref[i]))


def test_rms_scale_matches_oracle(gpu):
    lib, device, torch = gpu
    for M, K in [(1, 8), (5, 2048), (32, 8192), (7, 40)]:
        x = wl.make_x(M, K, 2300 + M, 0, 0)
        x[0, :] = 0                                   # a row of zeros: eps alone
        out = torch.empty(M, dtype=torch.float32, device="cuda")
        lib.rms_scale(device.to_device(x), M, K, 1e-5, out)
        torch.cuda.synchronize()
        ref = glue.rms_scale(bf16_bits_to_f32(x).astype(np.float64), 1e-5)
        assert np.max(np.abs(out.cpu().numpy() - ref) / ref) <= 1e-5


def test_fused_call_argument_checks(gpu):
    lib, device, torch = gpu
    p = wl.make_problem(wl.ProjShape("q", 256, 200, 32, 8, 2, 2.0), 2400, 0, 0)
    proj = device.upload_problem(p)
    x = device.to_device(wl.make_x(4, 256, 2400, 0, 0))
    y = device.alloc_y(4, 200, 0)
    ws = device.alloc_workspace([proj], 4)
    with pytest.raises(lib.MloraError):              # pair operation with N % 64 != 0
        lib.LayerPlanFused([proj], [lib.Epilogue(pair_op=lib.PAIR_SWIGLU)], [x], [y], None, 4, 0, ws).run()
    with pytest.raises(lib.MloraError):              # rotary tables missing
        lib.LayerPlanFused([proj], [lib.Epilogue(pair_op=lib.PAIR_ROPE)], [x], [y], None, 4, 0, ws).run()
    with pytest.raises(lib.MloraError):              # unknown operation
        lib.LayerPlanFused([proj], [lib.Epilogue(pair_op=7)], [x], [y], None, 4, 0, ws).run()
    with pytest.raises(lib.MloraError):              # more than 16 projections
        ys = [device.alloc_y(4, 200, 0) for _ in range(17)]
        lib.LayerPlanFused([proj] * 17, [lib.Epilogue()] * 17, [x] * 17, ys, None, 4, 0, ws).run()
