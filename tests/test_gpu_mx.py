"""GPU parity of the MX block quantiser (model_mx_quantize, through the C boundary) against the
CPU oracle: bit for bit (every step of Q(x) is exact in binary32)."""
import ctypes as C

import numpy as np
import pytest

import oracle.mx_oracle as mxo
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ae():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2602_17681_amd import binding
    return binding


def _run(ae, x32, block, dtype, inplace=False):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).cuda()
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    q = t if inplace else torch.full_like(t, float("nan"))
    rows, d = x32.shape
    ae.model_mx_quantize(t, q, rows, d, block)
    torch.cuda.synchronize()
    return q.float().cpu().numpy()


def _same_bits(a, o):
    """Bit for bit, except the sign of a zero result, which Eq. (1) does not define (the kernel keeps the
    input's sign, as an FP4 code would; the oracle returns -0 for small negative values and +0 for -0)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    o = np.ascontiguousarray(o, dtype=np.float32)
    nz = o != 0.0
    return np.array_equal(a, o) and np.array_equal(a.view(np.uint32)[nz], o.view(np.uint32)[nz])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,d,block", [(1, 32, 32), (37, 4096, 32), (513, 2048, 32), (64, 5120, 32), (129, 1024, 16),
                                          (33, 1024, 64), (7, 96, 8), (5, 12, 4), (9, 6, 2), (3, 90, 3), (11, 160, 160)])
def test_matches_oracle_bit_for_bit(ae, dtype, rows, d, block):
    x = wl.make_activations(rows, d, seed=rows + d + block, bf16=dtype == "bf16")
    got = _run(ae, x, block, dtype)
    want = mxo.mx_quantize(x.astype(np.float64), block).astype(np.float32)
    assert np.array_equal(want.astype(np.float64), mxo.mx_quantize(x.astype(np.float64), block))   # the result is a binary32 (and bf16) value
    assert _same_bits(got, want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_special_blocks(ae, dtype):
    """All-zero blocks, ties of every kind, values on the grid, clipping, very small and very large blocks."""
    rows = []
    rows.append(np.zeros(32))
    rows.append(np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0] * 4) * np.repeat([1, -1, 1, -1], 8))       # ties, max 6: s = 1
    rows.append(np.array([7.0, 6.5, 7.99, -7.5] + [0.5, 1, 1.5, 2, 3, 4, 6] * 4))                                   # clipping in (6, 8)
    rows.append(np.array([2.0 ** -130, 2.0 ** -133, -(2.0 ** -131)] + [0.0] * 29))                                   # scale exponent below -127
    rows.append(np.array([3.0e38, -1.0e38, 2.5e38, 1e30] + [1e37] * 28))                                            # near the top of binary32
    rows.append(np.array([1.0e-40, -3.0e-41] + [0.0] * 30))                                                          # subnormal block
    rows.append(np.array([10.0, 1.0] * 16))
    x = np.stack(rows).astype(np.float32)
    if dtype == "bf16":
        x = wl.round_to_bf16(x)
    got = _run(ae, x, 32, dtype)
    want = mxo.mx_quantize(x.astype(np.float64), 32).astype(np.float32)
    assert _same_bits(got, want)
    # the paper's worked example (block size 2): [10, 1, .5, .5] and its rotation [6, 4.5, 5, 4.5]
    ex = np.array([[10, 1, 0.5, 0.5], [6, 4.5, 5, 4.5]], dtype=np.float32)
    assert np.array_equal(_run(ae, ex, 2, dtype), [[8, 1, 0.5, 0.5], [6, 4, 4, 4]])


def test_in_place_idempotent_and_empty(ae):
    import torch
    x = wl.make_activations(257, 2048, seed=5, bf16=True)
    once = _run(ae, x, 32, "bf16")
    assert _same_bits(_run(ae, x, 32, "bf16", inplace=True), once)
    assert _same_bits(_run(ae, once, 32, "bf16"), once)                      # Q(Q(x)) = Q(x)
    t = torch.zeros(64, device="cuda")
    assert ae.lib.model_mx_quantize(C.c_void_p(t.data_ptr()), C.c_void_p(t.data_ptr()), 0, 64, 32, 0, None) == 0   # no rows: nothing to do
    for rows, d, block in ((1, 64, 0), (1, 0, 32), (1, 48, 32), (-1, 64, 32)):
        assert ae.lib.model_mx_quantize(C.c_void_p(t.data_ptr()), C.c_void_p(t.data_ptr()), rows, d, block, 0, None) == -1
    assert ae.lib.model_mx_quantize(None, C.c_void_p(t.data_ptr()), 1, 64, 32, 0, None) == -1
    assert ae.lib.model_mx_quantize(C.c_void_p(t.data_ptr()), C.c_void_p(t.data_ptr()), 1, 64, 32, 7, None) == -1


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_full_size_sampled_rows(ae, dtype):
    """The launch bench.py times (65 536 tokens x 4 096 channels, blocks of 32): 512 sampled rows against the oracle,
    and properties that hold for every element: idempotence, scaled magnitudes on the grid."""
    import torch
    rows, d = 65536, 4096
    gen = torch.Generator(device="cuda").manual_seed(17)
    x = torch.randn(rows, d, device="cuda", generator=gen) * torch.exp(torch.randn(1, d, device="cuda", generator=gen))
    x[:, ::509] *= 100.0
    x = x.to(torch.bfloat16 if dtype == "bf16" else torch.float32).contiguous()
    q = torch.empty_like(x)
    ae.model_mx_quantize(x, q, rows, d, 32)
    q2 = torch.empty_like(x)
    ae.model_mx_quantize(q, q2, rows, d, 32)
    torch.cuda.synchronize()
    assert torch.equal(q, q2)
    pick = np.random.default_rng(3).choice(rows, size=512, replace=False)
    pick.sort()
    idx = torch.from_numpy(pick).cuda()
    xs = x[idx].float().cpu().numpy()
    want = mxo.mx_quantize(xs.astype(np.float64), 32).astype(np.float32)
    assert _same_bits(q[idx].float().cpu().numpy(), want)
    # every block: quantised magnitudes divided by the block's scale lie on the E2M1 grid
    qb = q.float().view(-1, 32)
    amax = x.float().view(-1, 32).abs().amax(dim=1, keepdim=True)
    s = torch.exp2(torch.floor(torch.log2(amax.double())) - 2).float()
    ratio = (qb.abs() / s).flatten()
    grid = torch.tensor([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], device="cuda")
    assert bool(torch.isin(ratio, grid).all())
