"""CPU-only checks of the C-ABI library: it loads, exports every function the header declares,
sizes blobs and workspaces as documented, and rejects bad arguments on the host before any
launch (so none of these calls touches a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_2604_18655_amd as lib
from paper_2604_18655_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, EINVAL, ESHAPE, EALIGN, EWORKSPACE = 0, -1, -2, -3, -4


def header_functions():
    names = set()
    for header in ("mlora_w4.h", "mlora_tree_attention.h", "mlora_ds2d.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(mlora_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_function():
    cdll = lib.load_library()
    names = header_functions()
    assert set(names) == set(lib.exported_symbols)
    for name in names:
        assert getattr(cdll, name) is not None


def test_strerror_covers_all_codes():
    texts = {lib.strerror(c) for c in range(0, -7, -1)}
    assert len(texts) == 7 and "unknown" not in " ".join(texts)
    assert "unknown" in lib.strerror(-99)


def test_blob_bytes():
    # codes: ceil(N/64) tiles x K/32 steps x 1 KiB; scales: tiles x K/group x 128 B; 16 KiB slack
    slack = 16384
    assert lib.blob_bytes(256, 256, 32) == 4 * 8 * 1024 + 4 * 8 * 128 + slack
    assert lib.blob_bytes(256, 200, 64) == 4 * 8 * 1024 + 4 * 4 * 128 + slack
    assert lib.blob_bytes(2048, 8192, 32) == 8192 * 2048 // 2 + 8192 * 64 * 2 + slack
    for bad in [(100, 64, 32), (256, 64, 16), (256, 0, 32), (0, 64, 32), (64, 64, 32)]:
        assert lib.blob_bytes(*bad) == 0


def proj(K=256, N=64, group=32, blob=0x1000, n_ad=2, rank=8, a=0x2000, b=0x3000, alpha=1.0):
    return binding._ProjStruct(K, N, group, blob, n_ad, rank, a, b, alpha)


def test_workspace_bytes():
    """Size = 256 (status header) + 2 * max(counters, data), each rounded up to 256 bytes: the
    counters grow from the front, the data sits against the end, and with this size no call's
    counters can meet another call's data in a workspace that fits both."""
    cdll = lib.load_library()

    def need(ctrl, data):
        r = lambda v: (v + 255) // 256 * 256
        return 256 + 2 * max(r(ctrl), r(data))

    lines = lambda n_proj, part: (16 * n_proj + part) * 128    # 16 copies of a shrink counter per projection
    p = proj(K=2048, rank=16)
    # K/1024 = 2 chunks (at most 16) x M x rank16 x 4 bytes, rounded up to 256
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 8) == need(lines(1, 0), 2 * 8 * 16 * 4)
    p = proj(K=256, rank=8)
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 3) == need(lines(1, 0), 256)
    # K = 16384 = 8 units of 2048 inputs: 7 fp32 partial tiles [m_pad = 64][64] per tile of columns
    p = proj(K=16384, rank=64)
    # (+ one counter line per (tile, row chunk) of a split-K projection: 1 tile x 1 chunk)
    # (33 rows and more, chunks of 64 rows: a launch this small is cut further, here into 32
    # units of 4 x 128 inputs; the wide kernel's shrink step works on chunks of 2048 inputs where K
    # is above 4096 and leaves 8 chunks of partial sums)
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 64) == need(lines(1, 1), 8 * 64 * 64 * 4 + 31 * 1 * 64 * 64 * 4)
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 40) == need(lines(1, 1), 8 * 40 * 64 * 4 + 31 * 1 * 64 * 64 * 4)
    # (17 to 32 rows, a short launch: two chunks of 16 rows, 8 units of 2048 inputs, a shrink block
    # per row with at most 4 K chunks)
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 24) == need(lines(1, 2), 4 * 24 * 64 * 4 + 7 * 1 * 32 * 64 * 4)
    # a launch of the 64-row kernel with 80 to 240 base blocks gets K units of 8 x 128 inputs:
    # K = 3072, N = 8192 (128 tiles = 32 blocks of columns), 128 rows (2 chunks) -> 3 units
    p = proj(K=3072, N=8192, group=64, rank=16)
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 128) == need(lines(1, 128 * 2), 3 * 128 * 16 * 4
                                                                     + 2 * 128 * 128 * 64 * 4)
    p = proj(K=4096, N=200, n_ad=0, rank=0, a=None, b=None)
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 5) == need(lines(1, 4), 1 * 4 * 16 * 64 * 4)
    p = proj(n_ad=0, rank=0, a=None, b=None)
    assert cdll.mlora_w4_workspace_bytes(C.byref(p), 1, 8) == 0
    # several projections in one launch: 16 counter lines each
    arr = (binding._ProjStruct * 3)(proj(K=2048, rank=16), proj(K=256, rank=8), proj(K=2048, rank=16))
    assert cdll.mlora_w4_workspace_bytes(arr, 3, 8) == need(lines(3, 0), 2 * (2 * 8 * 16 * 4) + 256)
    # unsupported shapes and row counts have no size
    assert cdll.mlora_w4_workspace_bytes(C.byref(proj(K=100)), 1, 8) == 0
    assert cdll.mlora_w4_workspace_bytes(C.byref(proj()), 1, 4097) == 0


def test_layer_step_plan_names_the_kernel_family():
    """Blocks of one column tile up to 16 rows and for short launches of 17 to 32 rows; blocks of
    four column tiles from 33 rows on, and at 17 to 32 rows once a launch has 300 such blocks."""
    cdll = lib.load_library()
    info = (C.c_int32 * 5)()

    def plan(arr, n, M):
        assert cdll.mlora_w4_layer_step_plan(arr, n, M, info) == OK
        return list(info)

    one = (binding._ProjStruct * 1)(proj(K=2048, N=2048, rank=16))
    assert plan(one, 1, 8)[:3] == [1, 0, 16]
    assert plan(one, 1, 32)[:3] == [1, 0, 16]          # a short launch: two chunks of 16 rows
    seven = (binding._ProjStruct * 7)(*[proj(K=2048, N=n, rank=16) for n in (2048, 512, 512, 2048, 8192, 8192, 2048)])
    assert plan(seven, 7, 32)[:3] == [1, 0, 32]         # a whole layer: one chunk of 32 rows
    assert plan(one, 1, 33)[:3] == [1, 1, 64]
    many = (binding._ProjStruct * 130)(*[proj(K=2048, N=2048, rank=16) for _ in range(130)])
    got = plan(many, 130, 32)                           # 128 + 2 projections: two launches
    assert got[:3] == [2, 1, 32] and got[4] == 8
    assert plan(many, 130, 16)[:3] == [2, 0, 16]
    mixed = (binding._ProjStruct * 2)(proj(K=2048, group=32, rank=16), proj(K=2048, group=64, rank=16))
    assert plan(mixed, 2, 16)[0] == 1 and plan(mixed, 2, 17)[0] == 2   # group size changes
    assert cdll.mlora_w4_layer_step_plan(one, 1, 0, info) == ESHAPE
    assert cdll.mlora_w4_layer_step_plan(one, 0, 8, info) == EINVAL
    assert cdll.mlora_w4_layer_step_plan(one, 1, 8, None) == EINVAL


def test_workspace_init_rejects_bad_arguments():
    cdll = lib.load_library()
    assert cdll.mlora_w4_workspace_init(None, 0, None) == OK
    assert cdll.mlora_w4_workspace_init(None, 256, None) == EINVAL
    assert cdll.mlora_w4_workspace_init(0x7010, 256, None) == EALIGN


def call_linear(p, x=0x4000, rows=0x5000, M=4, y=0x6000, y_dtype=0, ws=0x7000, ws_bytes=1 << 20):
    return lib.load_library().mlora_w4_linear(C.byref(p), x, rows, M, y, y_dtype, ws, ws_bytes, None)


def test_linear_rejects_bad_arguments_before_launch():
    assert call_linear(proj(K=100)) == ESHAPE
    assert call_linear(proj(K=192)) == ESHAPE                 # K % 128
    for K in (32, 64, 96):                                     # multiples of the MFMA step, not of 128
        assert call_linear(proj(K=K)) == ESHAPE
        assert lib.blob_bytes(K, 64, 32) == 0
    assert call_linear(proj(group=48)) == ESHAPE
    assert call_linear(proj(N=0)) == ESHAPE
    assert call_linear(proj(rank=12)) == ESHAPE
    assert call_linear(proj(rank=136)) == ESHAPE
    assert call_linear(proj(n_ad=1025)) == ESHAPE
    assert call_linear(proj(), M=4097) == ESHAPE
    assert call_linear(proj(), M=-1) == ESHAPE
    assert call_linear(proj(blob=None)) == EINVAL
    assert call_linear(proj(a=None)) == EINVAL
    assert call_linear(proj(), x=None) == EINVAL
    assert call_linear(proj(), y=None) == EINVAL
    assert call_linear(proj(), y_dtype=2) == EINVAL
    assert call_linear(proj(blob=0x1008)) == EALIGN
    assert call_linear(proj(b=0x3004)) == EALIGN
    assert call_linear(proj(), x=0x4002) == EALIGN
    assert call_linear(proj(), ws=0x7010) == EALIGN           # workspace wants 256 bytes
    assert call_linear(proj(), ws=None) == EWORKSPACE
    assert call_linear(proj(), ws_bytes=16) == EWORKSPACE
    assert call_linear(proj(), M=0) == OK                     # empty call: nothing to launch
    assert lib.load_library().mlora_w4_linear(None, 1, 1, 1, 1, 0, 1, 1, None) == EINVAL


def test_layer_step_rejects_shared_outputs_and_bad_counts():
    cdll = lib.load_library()
    arr = (binding._ProjStruct * 2)(proj(), proj())
    xs = (C.c_void_p * 2)(0x4000, 0x4000)
    ys = (C.c_void_p * 2)(0x6000, 0x6000)
    assert cdll.mlora_w4_layer_step(arr, 2, xs, ys, 0x5000, 4, 0, 0x7000, 1 << 20, None) == EINVAL
    ys = (C.c_void_p * 2)(0x6000, 0x8000)
    assert cdll.mlora_w4_layer_step(arr, 0, xs, ys, 0x5000, 4, 0, 0x7000, 1 << 20, None) == EINVAL
    assert cdll.mlora_w4_layer_step(arr, 2, None, ys, 0x5000, 4, 0, 0x7000, 1 << 20, None) == EINVAL


def test_index_range_guard_refuses_the_whole_call_before_any_launch():
    """A projection with 2^16 column tiles is beyond the exact range of the kernels' block-index
    division.  It sits in the SECOND launch of the call (after 128 ordinary projections): the
    call is refused as a whole on the host, nothing is enqueued (all pointers here are fake)."""
    cdll = lib.load_library()
    n = 130
    arr = (binding._ProjStruct * n)(*[proj() for _ in range(n)])
    arr[129] = proj(N=1 << 22)
    xs = (C.c_void_p * n)(*[0x4000] * n)
    ys = (C.c_void_p * n)(*[0x100000 + 0x1000 * i for i in range(n)])
    assert cdll.mlora_w4_layer_step(arr, n, xs, ys, 0x5000, 4, 0, 0x7000, 1 << 40, None) == ESHAPE
    assert cdll.mlora_w4_workspace_bytes(arr, n, 4) == 0


def test_workspace_status_and_spin_limit_hooks():
    cdll = lib.load_library()
    assert cdll.mlora_w4_workspace_status(None, None, None) == EINVAL
    old = lib.debug_spin_limit(7)
    assert lib.debug_spin_limit(-1) == 7                      # negative: back to the default
    assert lib.debug_spin_limit(old) == old


def test_prepack_unpack_group_rows_reject_bad_arguments():
    cdll = lib.load_library()
    assert cdll.mlora_w4_prepack(256, 64, 32, None, 0x1000, 0x2000, None) == EINVAL
    assert cdll.mlora_w4_prepack(256, 64, 33, 0x1000, 0x1000, 0x2000, None) == ESHAPE
    assert cdll.mlora_w4_prepack(256, 64, 32, 0x1001, 0x1000, 0x2000, None) == EALIGN
    p = proj()
    assert cdll.mlora_w4_unpack(C.byref(p), None, None, None) == EINVAL
    assert cdll.mlora_w4_unpack(None, 0x1000, None, None) == EINVAL
    assert cdll.mlora_group_rows(0x1000, 4, 0, 0x1000, 0x1000, 0x1000, 0x1000, None) == ESHAPE
    assert cdll.mlora_group_rows(0x1000, 5000, 4, 0x1000, 0x1000, 0x1000, 0x1000, None) == ESHAPE
    assert cdll.mlora_group_rows(0x1000, 4, 4, None, 0x1000, 0x1000, 0x1000, None) == EINVAL
    assert cdll.mlora_group_rows(None, 4, 4, 0x1000, 0x1000, 0x1000, 0x1000, None) == EINVAL


def test_binding_raises_with_the_library_message():
    with pytest.raises(lib.MloraError) as e:
        binding._check(ESHAPE, "mlora_w4_linear")
    assert "unsupported shape" in str(e.value)


def tree_attn(**kw):
    f = dict(n_q_heads=8, n_kv_heads=2, head_dim=64, n_streams=2, rows_per_stream=4, scale=0.125,
             k_prefill=0x1000, v_prefill=0x2000, len_prefill=16, k_fprefix=0x3000, v_fprefix=0x4000, len_fprefix=4,
             k_stream=0x5000, v_stream=0x6000, cap_stream=32, len_stream=0x7000, k_new=0x8000, v_new=0x9000,
             parent=0xA000, is_forecast=0xB000)
    f.update(kw)
    return binding._TreeAttnStruct(**f)


def test_tree_attention_sizes_and_argument_checks():
    cdll = lib.load_library()
    t = tree_attn()
    # blocks of 64 keys, one chunk per block for short segments: 1 prefill + 1 prefix block for all
    # 8 rows x 4 heads per kv head, (1 + 1) blocks per stream for its 4 rows x 4 heads; 66 floats each
    want = ((1 + 1) * 2 * 32 + 2 * (1 + 1) * 2 * 16) * 66 * 4 + 256
    assert cdll.mlora_tree_attention_workspace_bytes(C.byref(t)) == want

    def call(t, q=0xC000, out=0xD000, dt=0, ws=0xE000, ws_bytes=1 << 30):
        return cdll.mlora_tree_attention(C.byref(t), q, out, dt, ws, ws_bytes, None)

    for bad in (dict(head_dim=96), dict(n_q_heads=7), dict(n_kv_heads=0), dict(rows_per_stream=65),
                dict(rows_per_stream=0), dict(n_streams=0), dict(n_streams=2000), dict(len_prefill=-1),
                dict(n_q_heads=36, n_kv_heads=2)):
        assert cdll.mlora_tree_attention_workspace_bytes(C.byref(tree_attn(**bad))) == 0
        assert call(tree_attn(**bad)) == ESHAPE
    for bad in (dict(k_new=None), dict(parent=None), dict(k_prefill=None), dict(v_fprefix=None), dict(len_stream=None)):
        assert call(tree_attn(**bad)) == EINVAL
    assert call(tree_attn(k_prefill=None, v_prefill=None, len_prefill=0), ws_bytes=16) == EWORKSPACE   # an empty segment needs no pointer
    assert call(tree_attn(k_stream=0x5008)) == EALIGN
    assert call(tree_attn(parent=0xA002)) == EALIGN
    assert call(t, q=None) == EINVAL
    assert call(t, dt=3) == EINVAL
    assert call(t, out=0xD004) == EALIGN
    assert call(t, ws=None) == EWORKSPACE
    assert call(t, ws_bytes=want - 1) == EWORKSPACE
    assert call(t, ws=0xE010) == EALIGN
    assert cdll.mlora_tree_attention(None, 1, 1, 0, 1, 1, None) == EINVAL


def test_ds2d_rows_layout_and_argument_checks():
    """Host side of the DS2D step: row counts of the paper's worked example (Section 3.5: m = 2,
    branch (3, 2): 10 tokens, 30 rows; first step 1 + m rows), the layout against the input
    generators' own, and the descriptor checks (nothing is launched)."""
    import numpy as np
    from workloads.attention import ds2d_tree
    assert lib.ds2d_rows((3, 2), 2) == (10, 30)
    assert lib.ds2d_rows((), 2) == (1, 3)
    assert lib.ds2d_rows((2,), 3) == (3, 12)
    for branch in [(3, 2), (2, 2, 2), (4,), (1, 1, 1)]:
        parent, is_forecast, level = lib.ds2d_layout(branch, len(branch))
        p2, f2 = ds2d_tree(branch)
        assert parent == list(p2) and is_forecast == list(f2)
    parent, is_forecast, level = lib.ds2d_layout((3, 2), 2)
    assert level[:10] == [0, 1, 1, 1, 2, 2, 2, 2, 2, 2] and level[10:14] == [1, 2, 1, 2]
    with pytest.raises(lib.MloraError):
        lib.ds2d_rows((3, 2, 4), 3)                  # 1 + 3 + 6 + 24 tokens x 4 rows > 64
    with pytest.raises(lib.MloraError):
        lib.ds2d_rows((3, 2), 1)                     # more levels than forecast embeddings
    with pytest.raises(lib.MloraError):
        lib.ds2d_rows((17,), 1)
    d = lib.Ds2dStep(2, 2, (3, 2), (3, 2), 1000, lib.Y_BF16)
    # 2 streams x 30 rows x 1 slice of 4096 logits x 16 keys of 8 bytes
    assert d.workspace_bytes() == 2 * 30 * 1 * 16 * 8
    assert lib.Ds2dStep(1, 2, (3, 2), (3, 2), 128256, lib.Y_BF16).workspace_bytes() == 30 * 32 * 16 * 8
    assert lib.Ds2dStep(1, 2, (3, 2), (3, 2), 2, lib.Y_BF16).workspace_bytes() == 0     # vocab < b'
    assert lib.Ds2dStep(0, 2, (3, 2), (3, 2), 100, lib.Y_BF16).workspace_bytes() == 0
    assert lib.Ds2dStep(1, 2, (3, 2), (3, 2), 100, 7).workspace_bytes() == 0
    cdll = lib.load_library()
    fn = cdll.mlora_ds2d_step
    st = C.byref(d.struct)
    assert fn(st, None, 16, 16, 16, 16, 16, 16, 1 << 20, None) == EINVAL
    assert fn(st, 8, 16, 16, 16, 16, 16, 16, 1 << 20, None) == EALIGN
    assert fn(st, 16, 16, 16, 16, 16, 16, 16, 100, None) == EWORKSPACE
    assert fn(st, 16, 16, 16, 16, 16, 16, None, 0, None) == EWORKSPACE
