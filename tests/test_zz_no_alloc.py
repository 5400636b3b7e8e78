"""The allocation-free variant of the transformation-error entry point against the workspace-taking one.

model_transform_mse_static keeps its per-tile partial sums in a buffer built into the library's device code, so
the same kernels must give the same bits as model_transform_mse_elem with a caller workspace: checked on two calls
in a row on the shared buffer, the second with a smaller input (stale contents of the first must not leak), and on
a shape beyond the buffer, which must be refused without touching the GPU."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _inputs(torch, rows, d, seed, dtype):
    bf = dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    dev = lambda arr, t=td: torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda().to(t).contiguous()
    x = wl.make_activations(rows, d, seed=seed, bf16=bf)
    a, v, ainv = wl.make_transform(d, seed=seed, bf16=bf, kind="affine")
    return dev(x), dev(a), dev(v, torch.float32), dev(ainv)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_point_matches_workspace_entry_point(dtype):
    import torch
    from paper_2602_17681_amd import binding as ae
    block = 32
    for rows, d, seed in ((2048, 1024, 31), (512, 256, 32)):        # the second call is the smaller one
        x, a, v, ainv = _inputs(torch, rows, d, seed, dtype)
        shift = torch.empty(d, device="cuda")
        ae.model_inverse_shift(ainv, v, d, shift)
        ws = torch.full((ae.model_transform_mse_workspace(rows, d, ae.DTYPES[dtype]) // 4,), float("nan"), device="cuda")
        res = []
        for static in (False, True):
            yq = torch.full_like(x, float("nan"))
            eb = torch.full((d // block,), float("nan"), device="cuda")
            et = torch.full((1,), float("nan"), device="cuda")
            if static:
                ae.model_transform_mse_static(x, a, v, ainv, shift, rows, d, block, yq, eb, et)
            else:
                ae.model_transform_mse(x, a, v, ainv, shift, rows, d, block, yq, ws, eb, et, elem="fp4")
            torch.cuda.synchronize()
            res.append((yq.float().cpu().numpy(), eb.cpu().numpy(), et.cpu().numpy()))
        (yq0, eb0, et0), (yq1, eb1, et1) = res
        assert np.all(np.isfinite(eb1)) and np.all(np.isfinite(et1)) and et1[0] > 0
        assert np.array_equal(yq0, yq1) and np.array_equal(eb0, eb1) and np.array_equal(et0, et1)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2602_17681_amd import binding as ae
    t = torch.zeros(64, device="cuda")
    p = C.c_void_p(t.data_ptr())
    # 65 536 x 4 096 bf16 needs 256 tiles x 2 x 4 096 floats = 8 MiB of partial sums: beyond the built-in 4 MiB
    assert ae.model_transform_mse_workspace(65536, 4096, ae.AE_BF16) > (4 << 20)
    assert ae.lib.model_transform_mse_static(p, p, p, p, p, 65536, 4096, 32, 0, ae.AE_BF16, p, p, p, None) == -1
    assert "built-in" in ae.model_last_error()
    assert ae.lib.model_transform_mse_static(p, p, p, p, p, 256, 128, 32, 9, ae.AE_BF16, p, p, p, None) == -1
