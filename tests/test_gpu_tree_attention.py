"""GPU parity of masked tree attention over a segmented KV cache against the fp64 oracle, through
the C ABI.  fp32 output within 2e-4 of max|out_ref| (fp32 accumulation, weights carried as two
bf16 halves: observed ~1e-6), bf16 output within 5e-3 (output rounding)."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

TOL, TOL_F32 = 5e-3, 2e-4


def gpu_attention(gpu, inp, out_dtype, Hq, Hkv, D):
    lib, device, torch = gpu
    dev = lambda a: device.to_device(a) if a.size else None
    t = lib.TreeAttention(Hq, Hkv, D, inp.n_streams, inp.rows_per_stream, inp.scale,
                          dev(inp.k_prefill), dev(inp.v_prefill), dev(inp.k_fprefix), dev(inp.v_fprefix),
                          dev(inp.k_stream), dev(inp.v_stream), torch.from_numpy(inp.len_stream).cuda(),
                          dev(inp.k_new), dev(inp.v_new), torch.from_numpy(inp.parent).cuda(),
                          torch.from_numpy(inp.is_forecast).cuda(),
                          inp.k_prefill.shape[1], inp.k_fprefix.shape[1], inp.k_stream.shape[2])
    M = inp.q.shape[0]
    out = torch.full((M, Hq, D), -5, dtype=torch.float32 if out_dtype == lib.Y_FP32 else torch.int16, device="cuda")
    ws = torch.empty(max(t.workspace_bytes(), 256), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                   # the workspace needs no initialisation: hand in garbage
    t.run(device.to_device(inp.q), out, out_dtype, ws)
    torch.cuda.synchronize()
    return device.y_to_numpy(out.reshape(M, Hq * D)).reshape(M, Hq, D)


def check(gpu, inp, Hq, Hkv, D, tag):
    lib = gpu[0]
    ref = oracle.tree_attention(inp.q, inp.k_prefill, inp.v_prefill, inp.k_fprefix, inp.v_fprefix,
                                inp.k_stream, inp.v_stream, inp.len_stream, inp.k_new, inp.v_new,
                                inp.parent, inp.is_forecast, inp.n_streams, inp.scale)
    o32 = gpu_attention(gpu, inp, lib.Y_FP32, Hq, Hkv, D)
    o16 = gpu_attention(gpu, inp, lib.Y_BF16, Hq, Hkv, D)
    scale = np.max(np.abs(ref))
    e32, e16 = float(np.max(np.abs(o32 - ref)) / scale), float(np.max(np.abs(o16 - ref)) / scale)
    print(f"{tag}: fp32-out err {e32:.2e}  bf16-out err {e16:.2e}", flush=True)
    assert e32 <= TOL_F32 and e16 <= TOL, tag
    # per row as well: a row that only sees a few keys must be as good as one that sees thousands
    row_err = np.max(np.abs(o32 - ref), axis=(1, 2)) / np.maximum(np.max(np.abs(ref), axis=(1, 2)), 1e-30)
    assert float(row_err.max()) <= 5 * TOL_F32, (tag, int(row_err.argmax()))
    assert np.array_equal(o32, gpu_attention(gpu, inp, lib.Y_FP32, Hq, Hkv, D))     # reproducible bit for bit
    return o32


@pytest.mark.parametrize("seed,tree,S,Hq,Hkv,D,Lp,Lf,cap", [
    (0, "ds2d32", 1, 8, 2, 64, 200, 10, 70),        # the paper's 30-row step, ragged segment lengths
    (1, "chain4", 8, 32, 8, 64, 2048, 0, 128),      # 8 streams x 4 rows, 1B-like heads, no forecast prefix
    (2, "random9", 3, 4, 4, 128, 65, 3, 64),        # head_dim 128, one query head per kv head, a chunk boundary + 1
    (3, "ds2d221", 5, 12, 2, 64, 0, 7, 0),          # no prefill, no stream cache: prefix and the step's rows only
    (4, "random64", 2, 6, 3, 128, 300, 64, 129),    # 64 rows per stream (the most), 2 heads per kv head
    (5, "chain1", 16, 8, 1, 64, 1000, 0, 33),       # one row per stream, 8 query heads on one kv head
    (6, "chain4", 2, 8, 4, 64, 5000, 130, 300),     # three chunks of keys per block, a last block with one; 5 chunks of stream keys in 2 blocks
])
def test_tree_attention_matches_oracle(gpu, seed, tree, S, Hq, Hkv, D, Lp, Lf, cap):
    rng = np.random.default_rng(seed)
    parent, fc = {"ds2d32": wl.ds2d_tree((3, 2)), "chain4": wl.chain_tree(4), "random9": wl.random_tree(9, rng),
                  "ds2d221": wl.ds2d_tree((2, 2, 1)), "random64": wl.random_tree(64, rng),
                  "chain1": wl.chain_tree(1)}[tree]
    inp = wl.make_attention_inputs(seed, S, parent, fc, Hq, Hkv, D, Lp, Lf, cap)
    check(gpu, inp, Hq, Hkv, D, f"{tree} S{S} Hq{Hq} Hkv{Hkv} D{D} Lp{Lp} Lf{Lf} cap{cap}")


def test_sharp_and_flat_softmax(gpu):
    """Keys ten times larger (one key takes nearly all the weight) and ten times smaller (nearly
    uniform weights), streams of length 0 and of full length side by side."""
    parent, fc = wl.ds2d_tree((2, 2))
    for k_std, seed in ((10.0, 20), (0.1, 21)):
        inp = wl.make_attention_inputs(seed, 4, parent, fc, 8, 2, 64, 130, 5, 64, len_stream=[0, 64, 1, 63], k_std=k_std)
        check(gpu, inp, 8, 2, 64, f"k_std {k_std}")


def test_streams_do_not_see_each_other_on_the_gpu(gpu):
    lib = gpu[0]
    parent, fc = wl.ds2d_tree((2, 1))
    a = wl.make_attention_inputs(30, 3, parent, fc, 8, 2, 64, 100, 4, 40, len_stream=[40, 17, 5])
    b = wl.make_attention_inputs(31, 3, parent, fc, 8, 2, 64, 100, 4, 40, len_stream=[3, 17, 29])
    R = len(parent)
    for name in ("k_prefill", "v_prefill", "k_fprefix", "v_fprefix"):
        setattr(b, name, getattr(a, name))
    for name in ("q", "k_new", "v_new"):
        getattr(b, name)[R:2 * R] = getattr(a, name)[R:2 * R]
    for name in ("k_stream", "v_stream"):
        getattr(b, name)[1] = getattr(a, name)[1]
    oa = gpu_attention(gpu, a, lib.Y_FP32, 8, 2, 64)
    ob = gpu_attention(gpu, b, lib.Y_FP32, 8, 2, 64)
    assert np.array_equal(oa[R:2 * R], ob[R:2 * R])
