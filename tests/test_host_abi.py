"""CPU-only checks of the C boundary: the library loads without a GPU, exports every
function the header declares, and its host-side planner (spec parser, shape inference,
parameter offsets, workspace sizing) agrees with the workload walker and the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle.ae_oracle as orc
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ae():
    from paper_2602_17681_amd import binding
    return binding


def test_every_declared_symbol_is_exported(ae):
    hdr = open(os.path.join(ROOT, "include", "aemodel.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(model_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(ae.SYMBOLS), declared ^ set(ae.SYMBOLS)
    raw = C.CDLL(os.path.join(ROOT, "paper_2602_17681_amd", "libaemodel.so"))
    for name in declared:
        assert hasattr(raw, name), name


def test_describe_matches_walker_and_oracle(ae):
    for name, cfg in wl.CONFIGS.items():
        for bn_mode in (0, 1):
            n, ic, oc, lat, ws = ae.model_describe(cfg["spec"], cfg["batch"], ae.DTYPES[cfg["dtype"]], bn_mode)
            ent, n2, ishape, oshape = wl.param_layout(cfg["spec"], bn_mode)
            assert (n, ic, oc) == (n2, ishape, oshape)
            assert orc.Net(cfg["spec"], 1, bn_mode).n_params == n
            assert ws > 0
    assert ae.model_describe(wl.CONFIGS["cfg5"]["spec"], 32, ae.AE_BF16)[3] == 4096
    # bf16 workspace is smaller than fp32 for the same network
    a = ae.model_describe(wl.CONFIGS["cfg2"]["spec"], 256, ae.AE_F32)[4]
    b = ae.model_describe(wl.CONFIGS["cfg2"]["spec"], 256, ae.AE_BF16)[4]
    assert b < a


@pytest.mark.parametrize("bad,code", [
    ("", -2), ("conv3:4", -2), ("in:3x4", -2), ("in:3x4x4,conv5:2", -2), ("in:3x5x5,conv3:2,pool2", -3),
    ("in:3x4x4,fc:5", -3), ("in:3x4x4,flatten,reshape:3x4x5", -3), ("in:3x4x4,conv3:0", -2), ("in:3x4x4,,relu", -2),
    ("in:3x4x4,foo", -2), ("in:3x4x4,relu", -2), ("in:3x4x4,up2,relu", -2), ("in:3x4x4,conv3:4,pool2,bn", -2),
    ("in:3x4x4,conv3:4x", -2), ("in:3x4x4,reshape:3x4x4", -2),
    # sizes that would overflow 32-bit arithmetic in the planner: refused before any step is built
    ("in:1x65536x65536,flatten,fc:8", -3), ("in:1x1x1,fc:8,reshape:65536x65536x1", -3), ("in:4x4x4,conv3:999999999", -3),
    ("in:4x4x4,conv3:9999999999", -2), ("in:999999999x999999999x999999999,conv3:4", -3), ("in:3x4x4", -2)])
def test_bad_specs(ae, bad, code):
    with pytest.raises(ae.AeError) as e:
        ae.model_describe(bad, 2)
    assert e.value.code == code
    assert ae.model_last_error()


def test_bad_arguments(ae):
    for args in [("in:3x4x4,conv3:4", 0, 0, 0), ("in:3x4x4,conv3:4", 2, 7, 0), ("in:3x4x4,conv3:4", 2, 0, 3)]:
        with pytest.raises(ae.AeError) as e:
            ae.model_describe(*args)
        assert e.value.code == -1
    assert ae.lib.model_describe(None, 1, 0, 0, None, None, None, None, None) == -1
    assert ae.lib.model_param_count(None, None) == -1
    assert ae.lib.model_loss_mse(None, None, 4, 0, None, None, None) == -1
    assert ae.lib.model_noise(0, 0, 1, 1, None, None) == -1
    ae.lib.model_destroy(None)   # no-op


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N > 1 exits with a message (before touching any GPU)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_host_only_argument_checks_of_the_widening_entry_points(ae):
    """Size and argument errors are reported on the host, before any GPU call."""
    n = C.c_int64()
    assert ae.lib.model_lu_workspace(48, 0, C.byref(n)) == -1 and "multiple of 32" in ae.model_last_error()
    assert ae.lib.model_lu_workspace(4096, 1, C.byref(n)) == 0 and n.value == 6 * 4096 * 4096 * 2 + 16384
    assert ae.lib.model_fold_workspace(4096, 4096, 4096, 128, 1, C.byref(n)) == 0 and n.value == (128 * 128 + 3 * 4096 * 4096) * 2 + 1024
    assert ae.lib.model_transform_mse_workspace(16384, 4096, 1, C.byref(n)) == 0 and n.value == 64 * 2 * 4096 * 4
    assert ae.lib.model_mx_quantize(None, None, 4, 64, 32, 1, None) == -1
    assert ae.lib.model_vol_penalty(None, 8, None, None, None) == -1
