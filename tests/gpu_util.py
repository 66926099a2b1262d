"""Helpers shared by the GPU parity tests: calls through the C ABI, comparisons with the oracle."""
import numpy as np

import oracle
import workloads as wl

TOL = 5e-3        # the stated gate, bf16 output (output rounding alone can reach 2^-8 = 3.9e-3)
TOL_F32 = 2e-4    # fp32 output: only fp32 accumulation-order error remains (observed ~1e-6)


def rel_err(y, ref):
    return float(np.max(np.abs(y - ref)) / np.max(np.abs(ref)))


def random_problem(seed, K, N, G, r, n_ad):
    shape = wl.ProjShape("t", K, N, G, r, n_ad, 2.0)
    return wl.make_problem(shape, 900 + seed, 0, 0)


def control_bytes(shapes, M):
    """Size of the status word + completion counters at the head of a workspace (one launch):
    16 counter lines of 128 bytes per projection and one more per (column tile, row chunk) of
    every projection whose K is cut into more than one unit of 2048 inputs."""
    rpc = 16 if M <= 16 else 32 if M < 33 else 64
    chunks = -(-M // rpc)
    n = sum(-(-s.N // 64) * chunks for s in shapes if -(-(s.K // 128) // 16) > 1)
    return 256 + (16 * len(shapes) + n) * 128


def assert_workspace_clean(gpu, ws, shapes, M):
    """After a call the status word is 0 (no block gave up waiting) and every counter is back
    at 0, so the next call can use the workspace as it is."""
    lib = gpu[0]
    assert lib.workspace_status(ws) == 0, "a block gave up waiting"
    n = min(control_bytes(shapes, M), ws.numel())
    assert int(ws[:n].count_nonzero().item()) == 0, "status word or completion counters not zero"


def run_linear(gpu, prob, x_bits, rows, y_dtype):
    lib, device, torch = gpu
    proj = device.upload_problem(prob)
    M = x_bits.shape[0]
    x = device.to_device(x_bits)
    ra = None if rows is None else torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda()
    y = device.alloc_y(M, prob.shape.N, y_dtype)
    ws = device.alloc_workspace([proj], max(M, 1))
    lib.linear(proj, x, ra, M, y, y_dtype, ws)
    torch.cuda.synchronize()
    if M > 0:
        assert_workspace_clean(gpu, ws, [prob.shape], M)
    return device.y_to_numpy(y)


def check_linear(gpu, prob, x_bits, rows, tag):
    G, alpha = prob.shape.group, prob.shape.alpha
    ref = oracle.linear(prob.wq, prob.scales, G, prob.lora_a, prob.lora_b, alpha, x_bits, rows)
    base = oracle.linear(prob.wq, prob.scales, G, prob.lora_a, prob.lora_b, alpha, x_bits, None)
    y16 = run_linear(gpu, prob, x_bits, rows, 0)
    y32 = run_linear(gpu, prob, x_bits, rows, 1)
    yb32 = run_linear(gpu, prob, x_bits, None, 1)
    e16, e32 = rel_err(y16, ref), rel_err(y32, ref)
    print(f"{tag}: bf16-out err {e16:.2e}  fp32-out err {e32:.2e}", flush=True)
    assert e16 <= TOL, tag
    assert e32 <= TOL_F32, tag
    assert rel_err(yb32, base) <= TOL_F32, tag
    delta_ref = ref - base
    if np.max(np.abs(delta_ref)) > 0:
        # the LoRA term on its own scale: a wrong adapter or a dropped alpha fails here
        assert float(np.max(np.abs((y32 - yb32) - delta_ref)) / np.max(np.abs(delta_ref))) <= TOL, tag
    return y16


def layer_on_gpu(gpu, probs, xs, rows, y_dtype):
    lib, device, torch = gpu
    projs = [device.upload_problem(p) for p in probs]
    cache = {}
    dxs = []
    for x in xs:
        if id(x) not in cache:
            cache[id(x)] = device.to_device(x)
        dxs.append(cache[id(x)])
    M = xs[0].shape[0]
    ra = torch.from_numpy(rows).cuda()
    ys = [device.alloc_y(M, p.shape.N, y_dtype) for p in probs]
    ws = device.alloc_workspace(projs, M)
    lib.layer_step(projs, dxs, ys, ra, M, y_dtype, ws)
    torch.cuda.synchronize()
    assert_workspace_clean(gpu, ws, [p.shape for p in probs], M)
    return [device.y_to_numpy(y) for y in ys]
