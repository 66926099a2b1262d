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
    epis, ys, sq_outs = [], [], []
    for p, sp in zip(probs, specs):
        pair = {"none": lib.PAIR_NONE, "rope": lib.PAIR_ROPE, "swiglu": lib.PAIR_SWIGLU}[sp.get("pair", "none")]
        sq_out = torch.full((M, -(-p.shape.N // 64)), -1.0, dtype=torch.float32, device="cuda") if sp.get("want_sq") else None
        sq_outs.append(sq_out)
        epis.append(lib.Epilogue(
            None if sp.get("row_scale") is None else dev_f32(torch, sp["row_scale"]), pair,
            None if sp.get("cos") is None else dev_f32(torch, sp["cos"]),
            None if sp.get("sin") is None else dev_f32(torch, sp["sin"]),
            None if sp.get("residual") is None else device.to_device(sp["residual"]),
            None if sp.get("sq_in") is None else dev_f32(torch, sp["sq_in"]),
            0 if sp.get("sq_in") is None else sp["sq_in"].shape[1], sp.get("sq_eps", 0.0), sq_out))
        n_out = p.shape.N // 2 if pair == lib.PAIR_SWIGLU else p.shape.N
        ys.append(device.alloc_y(M, n_out, y_dtype))
    ra = None if rows is None else torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda()
    ws = device.alloc_workspace(projs, M)
    lib.LayerPlanFused(projs, epis, dxs, ys, ra, M, y_dtype, ws).run()
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    for sp, sq in zip(specs, sq_outs):
        if sq is not None:
            sp["got_sq"] = sq.cpu().numpy().astype(np.float64)
    return [device.y_to_numpy(y) for y in ys]


def reference(probs, xs, rows, specs):
    out = []
    for p, x, sp in zip(probs, xs, specs):
        s = p.shape
        out.append(glue.fused_linear(p.wq, p.scales, s.group, p.lora_a, p.lora_b, s.alpha, x, rows,
                                     sp.get("row_scale"), sp.get("pair", "none"), sp.get("cos"), sp.get("sin"),
                                     sp.get("residual"), sp.get("sq_in"), sp.get("sq_eps", 0.0)))
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


@pytest.mark.parametrize("M", [5, 16, 30, 64])
def test_sums_of_squares_in_and_out(gpu, M):
    """RMSNorm without a kernel of its own: a projection leaves the sums of squares of its stored
    outputs per column tile, and the projection that reads those outputs scales its rows with
    them.  The sums are compared with the squares of the very outputs the device stored, the
    consumer with the oracle fed with the device's sums."""
    rng = np.random.default_rng(40 + M)
    K = 512
    pa = wl.make_problem(wl.ProjShape("o", K, 200, 32, 16, 3, 2.0), 2600 + M, 0, 0)      # 4 tiles, the last one ragged
    pg = wl.make_problem(wl.ProjShape("gate", K, 64, 32, 8, 3, 2.0), 2600 + M, 0, 1)
    pu = wl.make_problem(wl.ProjShape("up", K, 64, 32, 8, 3, 2.0), 2600 + M, 0, 2)
    x = wl.make_x(M, K, 2600 + M, 0, 0)
    rows = rng.integers(-1, 3, M).astype(np.int32)
    res = f32_to_bf16_bits(rng.standard_normal((M, 200)).astype(np.float32))
    for y_dtype in (1, 0):                            # (bf16 last: its outputs are the next projection's x below)
        specs = [dict(residual=res, want_sq=True), dict(pair="swiglu", want_sq=True)]
        probs = [pa, wl.fuse_gate_up(pg, pu)]
        got = run_fused(gpu, probs, [x, x], rows, M, y_dtype, specs)
        for i in range(2):
            want = glue.tile_squares(got[i], 64 if i == 0 else 32)       # a SwiGLU tile stores 32 columns
            assert specs[i]["got_sq"].shape == want.shape
            assert np.max(np.abs(specs[i]["got_sq"] - want)) <= 1e-5 * np.max(want), (M, i, y_dtype)
    # consumer: a projection whose x are the 200 columns the first one stored (padded to K = 256 with zeros)
    sq = specs[0]["got_sq"].astype(np.float32)
    pc = wl.make_problem(wl.ProjShape("c", 256, 128, 32, 16, 3, 2.0), 2600 + M, 0, 3)
    x2 = np.zeros((M, 256), np.uint16)
    x2[:, :200] = f32_to_bf16_bits(got[0].astype(np.float32))
    spec = [dict(sq_in=sq, sq_eps=1e-5, pair="rope", cos=np.ones((M, 32), np.float32), sin=np.zeros((M, 32), np.float32))]
    ref = reference([pc], [x2], rows, spec)
    out = run_fused(gpu, [pc], [x2], rows, M, 1, spec)
    assert rel_err(out[0], ref[0]) <= TOL_F32
    # and the scale those sums give is the scale of the stored rows
    direct = glue.rms_scale(bf16_bits_to_f32(x2).astype(np.float64), 1e-5)
    assert np.max(np.abs(glue.scale_from_parts(sq, 256, 1e-5) / direct - 1)) <= 1e-5


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


def build_layer(gpu, seed, S, parent, is_forecast, Hq, Hkv, F, Lp, cap, n_ad=3, rank=8):
    """A decoder layer of hidden = 64 * Hq on the device plus every host tensor it was made from."""
    lib, device, torch = gpu
    from paper_2604_18655_amd.decoder import DecoderLayerStep
    D, H, KV = 64, 64 * Hq, 64 * Hkv
    R = len(parent)
    M = S * R
    mk = lambda name, K, N, i: wl.make_problem(wl.ProjShape(name, K, N, 32, rank, n_ad, 2.0), seed, 0, i)
    host = {"q": mk("q", H, H, 0), "k": mk("k", H, KV, 1), "v": mk("v", H, KV, 2), "o": mk("o", H, H, 3),
            "gate_up": wl.fuse_gate_up(mk("gate", H, F, 4), mk("up", H, F, 5)), "down": mk("down", F, H, 6)}
    dev = {k: device.upload_problem(p) for k, p in host.items()}
    inp = wl.make_attention_inputs(seed, S, parent, is_forecast, Hq, Hkv, D, Lp, 0, cap)
    dd = lambda a: device.to_device(a) if a.size else None
    k_new = torch.zeros((M, Hkv * D), dtype=torch.int16, device="cuda")
    v_new = torch.zeros((M, Hkv * D), dtype=torch.int16, device="cuda")
    att = lib.TreeAttention(Hq, Hkv, D, S, R, inp.scale, dd(inp.k_prefill), dd(inp.v_prefill), None, None,
                            dd(inp.k_stream), dd(inp.v_stream), torch.from_numpy(inp.len_stream).cuda(), k_new, v_new,
                            torch.from_numpy(inp.parent).cuda(), torch.from_numpy(inp.is_forecast).cuda(), Lp, 0, cap)
    rng = np.random.default_rng(seed)
    h = wl.make_x(M, H, seed, 0, 9)
    ang = glue.rope_angles(rng.integers(0, 3000, M))
    cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    rows = rng.integers(-1, n_ad, M).astype(np.int32)
    layer = DecoderLayerStep(dev["q"], dev["k"], dev["v"], dev["o"], dev["gate_up"], dev["down"], att,
                             device.to_device(h), dev_f32(torch, cos), dev_f32(torch, sin),
                             torch.from_numpy(rows).cuda(), M)
    return layer, host, inp, h, cos, sin, rows


def bits_of(t):
    return t.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("S,branch", [(2, (3, 2)), (8, None)])
def test_decoder_layer_every_stage_and_end_to_end(gpu, S, branch):
    """A whole decoder layer through the library (7 calls), every stage compared with the oracle
    fed with the very tensors the stage read on the device, and the final rows with the oracle's
    own chain (intermediates rounded to bf16 where the device stores bf16)."""
    lib, device, torch = gpu
    if branch is None:
        parent, fc = np.asarray([-1, 0, 0, 1], np.int32), np.zeros(4, np.uint8)
    else:
        parent, fc = wl.ds2d_tree(branch)
    Hq, Hkv, F = 4, 2, 512
    layer, host, inp, h, cos, sin, rows = build_layer(gpu, 3100 + S, S, parent, fc, Hq, Hkv, F, 96, 24)
    layer.run()
    torch.cuda.synchronize()
    assert lib.workspace_status(layer.ws) == 0
    M = S * len(parent)
    f64 = lambda bits: bf16_bits_to_f32(bits).astype(np.float64)
    lin = lambda key, x_bits, **kw: glue.fused_linear(host[key].wq, host[key].scales, 32, host[key].lora_a,
                                                      host[key].lora_b, 2.0, x_bits, rows, **kw)
    att = lambda q, k, v: oracle.tree_attention(q.reshape(M, Hq, 64), inp.k_prefill, inp.v_prefill, inp.k_fprefix,
                                                inp.v_fprefix, inp.k_stream, inp.v_stream, inp.len_stream,
                                                k.reshape(M, Hkv, 64), v.reshape(M, Hkv, 64), inp.parent,
                                                inp.is_forecast, S, inp.scale).reshape(M, Hq * 64)
    s1 = layer.s1.cpu().numpy()
    assert np.max(np.abs(s1 / glue.rms_scale(f64(h), 1e-5) - 1)) <= 1e-5
    q, k, v = bits_of(layer.q), bits_of(layer.k_new), bits_of(layer.v_new)
    rope = dict(row_scale=s1, pair_op="rope", cos=cos, sin=sin)
    assert rel_err(f64(q), lin("q", h, **rope)) <= TOL
    assert rel_err(f64(k), lin("k", h, **rope)) <= TOL
    assert rel_err(f64(v), lin("v", h, row_scale=s1)) <= TOL
    attn = bits_of(layer.attn)
    assert rel_err(f64(attn), att(q, k, v)) <= TOL
    h2 = bits_of(layer.h2)
    assert rel_err(f64(h2), lin("o", attn, residual_bits=h)) <= TOL
    sq2 = layer.sq2.cpu().numpy()                                    # left by the o projection, per column tile
    assert np.max(np.abs(sq2 - glue.tile_squares(f64(h2)))) <= 1e-5 * np.max(sq2)
    assert np.max(np.abs(glue.scale_from_parts(sq2, Hq * 64, 1e-5) / glue.rms_scale(f64(h2), 1e-5) - 1)) <= 1e-5
    act = bits_of(layer.act)
    assert rel_err(f64(act), lin("gate_up", h2, sq_in=sq2, sq_eps=1e-5, pair_op="swiglu")) <= TOL
    out = bits_of(layer.out)
    assert rel_err(f64(out), lin("down", act, residual_bits=h2)) <= TOL
    out_sq = layer.out_sq.cpu().numpy()                              # for the next layer's first normalisation
    assert np.max(np.abs(out_sq - glue.tile_squares(f64(out)))) <= 1e-5 * np.max(out_sq)

    # the oracle's own chain, end to end
    rb = lambda y: f32_to_bf16_bits(y.astype(np.float32))
    o_s1 = glue.rms_scale(f64(h), 1e-5)
    o_rope = dict(row_scale=o_s1, pair_op="rope", cos=cos, sin=sin)
    o_q, o_k, o_v = rb(lin("q", h, **o_rope)), rb(lin("k", h, **o_rope)), rb(lin("v", h, row_scale=o_s1))
    o_attn = rb(att(o_q, o_k, o_v))
    o_h2 = rb(lin("o", o_attn, residual_bits=h))
    o_act = rb(lin("gate_up", o_h2, row_scale=glue.rms_scale(f64(o_h2), 1e-5), pair_op="swiglu"))
    o_out = lin("down", o_act, residual_bits=o_h2)
    assert rel_err(f64(out), o_out) <= 2e-2
