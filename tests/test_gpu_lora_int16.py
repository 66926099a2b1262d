"""GPU parity of int16 LoRA stacks served through mlora_lora_int16_expand and the layer step
(through the C ABI) against oracle/lora_int16.py.  The expansion is integer work: bit-exact
against the base-256 digits.  The layer step then multiplies exact integers and sums in fp32: the
bars of the bf16 path (<= 5e-3 of max|y_ref| with bf16 outputs, <= 2e-4 with fp32 outputs) and the
LoRA term on its own scale."""
import numpy as np
import pytest

import oracle
from oracle import lora_int16 as oi
import workloads as wl
from gpu_util import TOL, TOL_F32, rel_err

pytestmark = pytest.mark.gpu


def _bf16_bits_of_ints(v):
    bits = wl.f32_to_bf16_bits(v.astype(np.float32))
    assert np.array_equal(wl.bf16_bits_to_f32(bits), v.astype(np.float32))      # exact by construction
    return bits


@pytest.mark.parametrize("K,N,r,n_ad", [(128, 64, 8, 3), (256, 136, 16, 5), (2048, 512, 32, 2)])
def test_expansion_is_the_digits_bit_for_bit(gpu, K, N, r, n_ad):
    lib, device, torch = gpu
    rng = np.random.default_rng(K + N)
    aq = rng.integers(-32768, 32768, (n_ad, r, K)).astype(np.int16)
    bq = rng.integers(-32768, 32768, (n_ad, N, r)).astype(np.int16)
    aq[0, 0, :4] = [-32768, 32767, -1, 0]
    bq[0, 0, :4] = [-32768, 32767, -1, 255]
    da, db = device.to_device(aq), device.to_device(bq)
    a4 = torch.full((n_ad, 4 * r, K), -1, dtype=torch.int16, device="cuda")
    b4 = torch.full((n_ad, N, 4 * r), -1, dtype=torch.int16, device="cuda")
    alpha = lib.lora_int16_expand(da, db, n_ad, r, K, N, 2.0, 3.0e-5, 7.0e-6, a4, b4)
    torch.cuda.synchronize()
    assert alpha == float(np.float32(2.0) * np.float32(3.0e-5) * np.float32(7.0e-6))
    ah, al = oi.digits(aq)
    bh, bl = oi.digits(bq)
    want_a = _bf16_bits_of_ints(np.concatenate([ah, ah, al, al], axis=1))
    want_b = _bf16_bits_of_ints(np.concatenate([65536 * bh, 256 * bl, 256 * bh, bl], axis=2))
    assert np.array_equal(a4.cpu().numpy().view(np.uint16), want_a)
    assert np.array_equal(b4.cpu().numpy().view(np.uint16), want_b)


def _run(gpu, proj, x, rows, M, N, y_dtype):
    lib, device, torch = gpu
    dx = device.to_device(x)
    y = device.alloc_y(M, N, y_dtype)
    ra = None if rows is None else torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda()
    ws = device.alloc_workspace([proj], M)
    lib.LayerPlan([proj], [dx], [y], ra, M, y_dtype, ws).run()
    torch.cuda.synchronize()
    assert lib.workspace_status(ws) == 0
    return device.y_to_numpy(y)


# (K, N, group, rank, adapters, rows): the tile blocks' short way out (4 * rank = 32), their general
# one (64), two chunks of 16 rows, and the wide blocks at 32 (long launch not needed: 33+) and 64 rows
@pytest.mark.parametrize("K,N,G,r,n_ad,M", [
    (256, 256, 32, 8, 8, 8),
    (2048, 512, 32, 16, 8, 8),
    (2048, 2048, 32, 16, 8, 32),
    (1024, 200, 64, 16, 5, 40),
    (4096, 1024, 128, 32, 6, 64),
])
def test_layer_step_with_int16_lora_matches_oracle(gpu, K, N, G, r, n_ad, M):
    lib, device, torch = gpu
    shape = wl.ProjShape("t", K, N, G, r, n_ad, 2.0)
    q = wl.make_problem_lora_int16(shape, 1700 + M, 0, 0)
    x = wl.make_x(M, K, 1700 + M, 0, 0)
    rows = np.random.default_rng(M + K).integers(-1, n_ad, size=M).astype(np.int32)
    proj = device.upload_problem_lora_int16(q)
    assert proj.rank == 4 * r
    ref = oi.linear(q.wq, q.scales, G, q.aq, q.s_a, q.bq, q.s_b, shape.alpha, x, rows)
    delta = oi.lora_delta(q.aq, q.s_a, q.bq, q.s_b, shape.alpha, x, rows)
    base = ref - delta
    y16 = _run(gpu, proj, x, rows, M, N, 0)
    y32 = _run(gpu, proj, x, rows, M, N, 1)
    yb32 = _run(gpu, proj, x, None, M, N, 1)
    assert rel_err(y16, ref) <= TOL, ("bf16", rel_err(y16, ref))
    assert rel_err(y32, ref) <= TOL_F32, ("fp32", rel_err(y32, ref))
    assert rel_err(yb32, base) <= TOL_F32, ("base", rel_err(yb32, base))
    assert np.max(np.abs(delta)) > 0
    assert np.max(np.abs((y32 - yb32) - delta)) <= TOL * np.max(np.abs(delta)), "lora term on its own scale"


def test_expand_argument_checks(gpu):
    lib, device, torch = gpu
    a = torch.zeros((1, 8, 64), dtype=torch.int16, device="cuda")
    b = torch.zeros((1, 64, 8), dtype=torch.int16, device="cuda")
    a4 = torch.zeros((1, 32, 64), dtype=torch.int16, device="cuda")
    b4 = torch.zeros((1, 64, 32), dtype=torch.int16, device="cuda")
    with pytest.raises(lib.MloraError):
        lib.lora_int16_expand(a, b, 1, 40, 64, 64, 1.0, 1.0, 1.0, a4, b4)      # 4 * rank above the maximum
    with pytest.raises(lib.MloraError):
        lib.lora_int16_expand(a, b, 1, 12, 64, 64, 1.0, 1.0, 1.0, a4, b4)      # rank not a multiple of 8
    with pytest.raises(lib.MloraError):
        lib.lora_int16_expand(a, b, 1, 8, 64, 64, 1.0, 0.0, 1.0, a4, b4)       # a scale must be positive
    with pytest.raises(lib.MloraError):
        lib.lora_int16_expand(a, None, 1, 8, 64, 64, 1.0, 1.0, 1.0, a4, b4)
