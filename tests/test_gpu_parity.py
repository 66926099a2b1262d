"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact for unpacked codes, dequantised weights and row grouping; outputs
within max|y - y_ref| / max|y_ref| <= 5e-3 (bf16 output) and a tighter bound for fp32 output.
"""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import (TOL, TOL_F32, assert_workspace_clean, check_linear, layer_on_gpu,
                      random_problem, rel_err, run_linear)

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------------------ unpack

@pytest.mark.parametrize("K,N,G", [(128, 64, 32), (256, 200, 64), (384, 17, 128), (2048, 512, 32)])
def test_unpack_bit_exact(gpu, K, N, G):
    lib, device, torch = gpu
    rng = np.random.default_rng(K + N)
    codes = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    codes[0, :16] = np.arange(-8, 8)                 # every code value, including -8
    codes[N - 1, K - 16:] = np.arange(7, -9, -1)
    scales = rng.uniform(1e-3, 3e-2, size=(N, K // G)).astype(np.float16).view(np.uint16)
    shape = wl.ProjShape("u", K, N, G, 8, 0, 1.0)
    prob = wl.Problem(shape, wl.pack_nibbles(codes), scales, None, None)
    proj = device.upload_problem(prob, with_lora=False)
    out_codes = torch.empty((N, K), dtype=torch.int8, device="cuda")
    out_w = torch.empty((N, K), dtype=torch.float32, device="cuda")
    lib.unpack(proj, out_codes, out_w)
    torch.cuda.synchronize()
    assert np.array_equal(out_codes.cpu().numpy(), oracle.unpack_codes(prob.wq))
    assert np.array_equal(out_w.cpu().numpy().astype(np.float64),
                          oracle.dequant(prob.wq, scales, G))


# ------------------------------------------------------------------------------ grouping

def gpu_group(gpu, rows, n_ad):
    lib, device, torch = gpu
    M = len(rows)
    ra = torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda() if M else \
        torch.zeros(1, dtype=torch.int32, device="cuda")
    perm = torch.full((max(M, 1),), -7, dtype=torch.int32, device="cuda")
    seg_a = torch.full((n_ad,), -7, dtype=torch.int32, device="cuda")
    seg_s = torch.full((n_ad + 1,), -7, dtype=torch.int32, device="cuda")
    n_seg = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    lib.group_rows(ra, M, n_ad, perm, seg_a, seg_s, n_seg)
    torch.cuda.synchronize()
    u = int(n_seg.item())
    return perm.cpu().numpy()[:M], seg_a.cpu().numpy(), seg_s.cpu().numpy(), u


def test_group_rows_bit_exact(gpu):
    rng = np.random.default_rng(5)
    cases = [rng.integers(-1, n_ad, size=M).astype(np.int32)
             for M, n_ad in [(1, 1), (8, 8), (128, 8), (64, 32), (257, 5), (33, 64), (4096, 1024),
                             (4096, 3), (100, 700)]]
    n_ads = [1, 8, 8, 32, 5, 64, 1024, 3, 700]
    for key in ("c1", "c3", "c3_interleaved", "c4_decode", "c4_prefill", "c5_up"):
        w = wl.WORKLOADS[key]
        cases.append(wl.make_rows(w.row_map, w.M, w.projs[0].n_adapters, w.cfg_id))
        n_ads.append(w.projs[0].n_adapters)
    cases += [np.full(16, -1, np.int32), np.zeros(0, np.int32), np.full(70, 3, np.int32)]
    n_ads += [4, 4, 4]
    for rows, n_ad in zip(cases, n_ads):
        perm, seg_a, seg_s, u = gpu_group(gpu, rows, n_ad)
        o_perm, o_seg_a, o_seg_s = oracle.group_rows(rows, n_ad)
        assert u == len(o_seg_a)
        assert np.array_equal(perm, o_perm)
        assert np.array_equal(seg_a[:u], o_seg_a)
        assert np.array_equal(seg_s[:u + 1], o_seg_s)


def test_group_rows_flags_out_of_range_index(gpu):
    for bad in (np.array([0, 4, 1], np.int32), np.array([-2, 0], np.int32)):
        _, _, _, u = gpu_group(gpu, bad, 4)
        assert u == -1
        with pytest.raises(ValueError):
            oracle.group_rows(bad, 4)


# ------------------------------------------------------------------------------ linear

def test_config1_tiny(gpu):
    w = wl.WORKLOADS["c1"]
    probs, xs, rows = wl.make_layer(w)
    y1 = check_linear(gpu, probs[0], xs[0], rows, "c1")
    y2 = run_linear(gpu, probs[0], xs[0], rows, 0)
    assert np.array_equal(y1, y2)                     # same inputs twice -> bit-identical


@pytest.mark.parametrize("K,N,G,r,n_ad,M", [
    (128, 64, 32, 8, 2, 1),         # smallest legal shape, one row
    (256, 200, 64, 8, 3, 5),        # ragged N (not a multiple of 16), rank below one MFMA block
    (640, 72, 128, 24, 4, 16),      # K/128 = 5 super-steps over 4 waves, rank 24
    (384, 136, 32, 16, 5, 17),      # one row into the second block of 16
    (1152, 96, 64, 64, 6, 33),      # first size of the 64-row kernel, rank 64
    (512, 64, 32, 128, 2, 9),       # maximum rank
    (4096, 128, 128, 16, 9, 70),    # K chunks in the shrink step, two row chunks
    (896, 136, 32, 24, 6, 24),      # 17-32 rows: one chunk of 32, 24 rows staged, odd super-steps
    (2560, 200, 64, 16, 11, 32),    # 17-32 rows: full chunk, more adapters than a tile has rows
    (768, 264, 128, 40, 4, 48),     # 33-63 rows: a partly empty chunk of 64
    (12288, 136, 32, 16, 3, 7),     # decode with 6 K units (more than the 4 of the common case)
    (16384, 72, 64, 8, 2, 12),      # decode with 8 K units, 9-16 rows
    (20480, 64, 128, 16, 2, 5),     # decode with 10 K units: the general way out
])
def test_ragged_shapes(gpu, K, N, G, r, n_ad, M):
    prob = random_problem(K + N + M, K, N, G, r, n_ad)
    rng = np.random.default_rng(M)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    rows = rng.integers(-1, n_ad, size=M).astype(np.int32)
    check_linear(gpu, prob, x, rows, f"K{K} N{N} G{G} r{r} a{n_ad} M{M}")


@pytest.mark.parametrize("K,N,G,r,n_ad,M", [
    (128, 64, 32, 8, 2, 64),        # one super-step, one tile (three spare waves), exactly one chunk
    (384, 200, 64, 24, 3, 65),      # ragged N inside the fourth tile, one row in the second chunk
    (640, 328, 128, 128, 5, 100),   # six tiles (two blocks of columns), maximum rank, odd super-steps
    (2304, 96, 32, 40, 7, 129),     # small launch: K cut into units, rank not a multiple of 16
    (512, 1024, 32, 16, 40, 200),   # more adapters than rows of a 16-row block, four full blocks
])
def test_wide_shapes(gpu, K, N, G, r, n_ad, M):
    """33 rows and more take the kernel with 64 x 256 blocks: ragged tiles, chunks and ranks."""
    prob = random_problem(K + N + M, K, N, G, r, n_ad)
    rng = np.random.default_rng(M)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    rows = rng.integers(-1, n_ad, size=M).astype(np.int32)
    check_linear(gpu, prob, x, rows, f"wide K{K} N{N} G{G} r{r} a{n_ad} M{M}")
    # rows grouped by adapter, all rows without adapter, no row index at all
    check_linear(gpu, prob, x, np.sort(rows), "wide, grouped rows")
    check_linear(gpu, prob, x, np.full(M, -1, np.int32), "wide, base only")
    y = run_linear(gpu, prob, x, None, 1)
    y_base = run_linear(gpu, prob, x, np.full(M, -1, np.int32), 1)
    assert np.array_equal(y, y_base)


@pytest.mark.parametrize("K,N,G,r,n_ad,M", [
    (256, 76810, 64, 24, 5, 23),      # 301 blocks of four tiles, ragged last tile, one stage of 8 k-steps
    (4352, 25605, 32, 16, 9, 19),     # 34 super-steps in 3 K units (11/12: odd, a half stage at the end), split-K sums
    (640, 77000, 128, 128, 3, 32),    # full chunk, maximum rank, group of 4 k-steps, 5 super-steps
    (1152, 77777, 32, 8, 40, 17),     # one row into the second block of 16, more adapters than rows
])
def test_wide_blocks_at_17_to_32_rows(gpu, K, N, G, r, n_ad, M):
    """Calls of 17 to 32 rows with 300 and more blocks of four column tiles run the kernel that
    shares the rows of x through LDS (chunks of 32 rows); smaller launches run one-tile blocks."""
    prob = random_problem(K + N + M, K, N, G, r, n_ad)
    rng = np.random.default_rng(M)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    rows = rng.integers(-1, n_ad, size=M).astype(np.int32)
    check_linear(gpu, prob, x, rows, f"wide32 K{K} N{N} G{G} r{r} a{n_ad} M{M}")


@pytest.mark.parametrize("K,N,G,r,n_ad,M", [
    (1024, 700, 32, 16, 5, 200),      # 4 chunks of 64 rows (the last with 8), 3 blocks of columns: a run of 8 is not full
    (2560, 2100, 64, 16, 9, 330),     # 6 chunks, 9 blocks of columns, several K units: runs of 8 plus a remainder
    (512, 130, 128, 8, 3, 1000),      # 16 chunks, one block of columns
])
def test_many_row_chunks(gpu, K, N, G, r, n_ad, M):
    """Calls with several row chunks lay their blocks out in runs of 8 with the chunk varying in
    steps of 8 (all chunks of a block of columns on one XCD): every (block, chunk) pair must be
    computed exactly once whatever the counts are."""
    prob = random_problem(K + N + M, K, N, G, r, n_ad)
    rng = np.random.default_rng(M)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    rows = rng.integers(-1, n_ad, size=M).astype(np.int32)
    check_linear(gpu, prob, x, rows, f"chunks K{K} N{N} G{G} r{r} a{n_ad} M{M}")


def test_wide_extreme_and_zero_scales(gpu):
    """The wide kernel keeps its accumulators in units of the current group's scale: scales that
    jump by many orders of magnitude between groups, and zero scales, must not disturb it."""
    K, N, G, M = 1024, 128, 32, 64
    rng = np.random.default_rng(5)
    codes = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    codes[::3] = 7
    codes[1::3] = -8
    groups = K // G
    sc = np.empty((N, groups), np.float16)
    sc[:, 0::4] = np.float16(0.5)
    sc[:, 1::4] = np.float16(6.1e-5)
    sc[:, 2::4] = np.float16(0.0)                 # dead groups: contribute exactly nothing
    sc[:, 3::4] = np.float16(2.0e-2)
    sc[5, :] = np.float16(0.0)                    # a column that is dead throughout
    sc[6, :3] = np.float16(0.0)                   # a column that starts dead
    sc[7, 0] = np.float16(8.0)                    # large then tiny
    shape = wl.ProjShape("e", K, N, G, 16, 2, 1.0)
    prob = wl.Problem(shape, wl.pack_nibbles(codes), sc.view(np.uint16),
                      wl.f32_to_bf16_bits(rng.standard_normal((2, 16, K)).astype(np.float32) / 32),
                      wl.f32_to_bf16_bits(rng.standard_normal((2, N, 16)).astype(np.float32)))
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, ::7] *= np.float32(1e-3)
    rows = rng.integers(-1, 2, size=M).astype(np.int32)
    check_linear(gpu, prob, wl.f32_to_bf16_bits(x), rows, "wide extreme")


def test_extreme_codes_and_scales(gpu):
    # all codes -8 / +7, large and tiny scales, x with large dynamic range
    K, N, G, M = 256, 64, 32, 4
    codes = np.full((N, K), -8, np.int8)
    codes[::2] = 7
    scales = np.full((N, K // G), np.float16(0.5).view(np.uint16), np.uint16)
    scales[:, 1::2] = np.float16(6.1e-5).view(np.uint16)
    shape = wl.ProjShape("e", K, N, G, 8, 1, 1.0)
    rng = np.random.default_rng(0)
    prob = wl.Problem(shape, wl.pack_nibbles(codes), scales,
                      wl.f32_to_bf16_bits(rng.standard_normal((1, 8, K)).astype(np.float32)),
                      wl.f32_to_bf16_bits(rng.standard_normal((1, N, 8)).astype(np.float32)))
    x = rng.standard_normal((M, K)).astype(np.float32) * np.float32(100.0)
    x[:, ::7] *= np.float32(1e-3)
    check_linear(gpu, prob, wl.f32_to_bf16_bits(x), np.array([0, -1, 0, 0], np.int32), "extreme")


def test_empty_call_is_a_no_op(gpu):
    lib, device, torch = gpu
    prob = random_problem(1, 128, 64, 32, 8, 2)
    proj = device.upload_problem(prob)
    x = torch.zeros((1, 128), dtype=torch.int16, device="cuda")
    y = torch.full((1, 64), 77, dtype=torch.int16, device="cuda")
    lib.linear(proj, x, None, 0, y, 0, None)
    torch.cuda.synchronize()
    assert int((y == 77).all().item()) == 1


def test_rows_sharing_an_adapter_match_single_row_calls(gpu):
    prob = random_problem(3, 512, 128, 32, 16, 4)
    rng = np.random.default_rng(3)
    x = wl.f32_to_bf16_bits(rng.standard_normal((12, 512)).astype(np.float32))
    rows = np.array([2, 2, 2, 0, 0, 1, 1, 1, 1, 3, -1, 2], np.int32)
    y = run_linear(gpu, prob, x, rows, 1)
    for m in range(12):
        y1 = run_linear(gpu, prob, x[m:m + 1], rows[m:m + 1], 1)
        assert rel_err(y1[0:1], y[m:m + 1]) <= 1e-5


@pytest.mark.parametrize("M", [5, 40, 72])
def test_layer_step_many_projections_mixed_groups(gpu, M):
    """More projections than one launch holds (16), group sizes mixed (33 rows and more: a launch
    per run of equal group size), with and without split K, some without adapters."""
    lib, device, torch = gpu
    rng = np.random.default_rng(100 + M)
    shapes = []
    for i in range(19):
        K = [256, 384, 2304, 128][i % 4]
        N = [64, 200, 96, 130][(i // 2) % 4]
        G = [32, 64, 128][i % 3] if i % 5 else 32
        r = [8, 16, 24, 64][i % 4]
        n_ad = 0 if i == 7 else 4
        shapes.append(wl.ProjShape(f"p{i}", K, N, G, r, n_ad, 1.5))
    probs = [wl.make_problem(s, 77, 0, i) for i, s in enumerate(shapes)]
    xs_by_k = {K: wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)) for K in {s.K for s in shapes}}
    xs = [xs_by_k[s.K] for s in shapes]
    rows = rng.integers(-1, 4, size=M).astype(np.int32)
    ys = layer_on_gpu(gpu, probs, xs, rows, 1)
    for p, x, y in zip(probs, xs, ys):
        ref = oracle.linear(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha, x,
                            rows if p.shape.n_adapters else None)
        assert rel_err(y, ref) <= TOL_F32, p.shape.name


def test_maximum_rows(gpu):
    """M = 4096, the most rows a call takes: 64 chunks of the wide kernel; oracle on sampled rows."""
    K, N, G, r, n_ad, M = 256, 136, 64, 16, 3, 4096
    prob = random_problem(4096, K, N, G, r, n_ad)
    rng = np.random.default_rng(4096)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    rows = rng.integers(-1, n_ad, size=M).astype(np.int32)
    y = run_linear(gpu, prob, x, rows, 1)
    sel = np.concatenate([np.arange(0, 70), rng.choice(M, 200, replace=False), np.arange(M - 70, M)])
    ref = oracle.linear(prob.wq, prob.scales, G, prob.lora_a, prob.lora_b, prob.shape.alpha,
                        np.ascontiguousarray(x[sel]), np.ascontiguousarray(rows[sel]))
    assert rel_err(y[sel], ref) <= TOL_F32


def test_workspace_reuse_and_graph_replay_match_first_call(gpu):
    """One workspace serves call after call (the counters reset themselves), eagerly and as a
    captured graph replayed several times with eager work in between: every result equals the
    first call's bit for bit."""
    lib, device, torch = gpu
    w = wl.WORKLOADS["c2"]
    probs, xs, rows = wl.make_layer(w, layer=1)
    projs = [device.upload_problem(p) for p in probs]
    cache, dxs = {}, []
    for x in xs:
        if id(x) not in cache:
            cache[id(x)] = device.to_device(x)
        dxs.append(cache[id(x)])
    M = w.M
    ra = torch.from_numpy(rows).cuda()
    ys = [device.alloc_y(M, p.shape.N, lib.Y_BF16) for p in probs]
    ws = device.alloc_workspace(projs, M)
    plan = lib.LayerPlan(projs, dxs, ys, ra, M, lib.Y_BF16, ws)

    def snapshot_and_clobber():
        torch.cuda.synchronize()
        assert_workspace_clean(gpu, ws, [p.shape for p in probs], M)
        out = [y.clone() for y in ys]
        for y in ys:
            y.fill_(-1)
        return out

    plan.run()
    first = snapshot_and_clobber()
    for _ in range(3):
        plan.run()
        again = snapshot_and_clobber()
        assert all(torch.equal(a, b) for a, b in zip(first, again))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            plan.run(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for i in range(4):
        graph.replay()
        again = snapshot_and_clobber()
        assert all(torch.equal(a, b) for a, b in zip(first, again)), f"replay {i}"
        plan.run()                                   # eager work between replays
        again = snapshot_and_clobber()
        assert all(torch.equal(a, b) for a, b in zip(first, again))
