"""ctypes binding of libaemodel.so: argument marshalling only.

Every function has the name and argument order of the C entry point it calls
(include/aemodel.h).  Tensors are torch tensors on the GPU; the binding passes
their data pointers and the current HIP stream and checks the status code.
Nothing is computed here and there is no fallback: if the library is missing the
import fails.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaemodel.so")

AE_F32, AE_BF16 = 0, 1
DTYPES = {"f32": AE_F32, "bf16": AE_BF16}
TORCH_DTYPE = {AE_F32: torch.float32, AE_BF16: torch.bfloat16}

SYMBOLS = [
    "model_describe", "model_create", "model_destroy", "model_param_count", "model_io_shape",
    "model_set_sample_offset", "model_forward", "model_backward", "model_loss_mse", "model_noise",
    "model_pnorm_awgn", "model_gen_bits", "model_count_errors", "model_monte_carlo", "model_num_steps", "model_step_info",
    "model_get_activation", "model_get_conv_output", "model_timing_enable", "model_set_overlap", "model_set_params_static", "model_set_inference", "model_set_recompute", "model_set_fused_backward", "model_calibrate_mfma", "model_mx_quantize", "model_mx_quantize_elem", "model_transform_mse_workspace",
    "model_transform_mse", "model_transform_mse_elem", "model_transform_mse_static", "model_inverse_shift", "model_lu_workspace", "model_lu_compose", "model_lu_backward", "model_vol_penalty", "model_lu_inverse_workspace", "model_lu_inverse", "model_lu_compose_batch", "model_lu_backward_batch", "model_lu_inverse_batch", "model_lu_timing", "model_qr_workspace", "model_qr_squarings", "model_qr_compose", "model_qr_backward", "model_qr_inverse", "model_fold_workspace", "model_fold_linear", "model_fold_embedding", "model_timing_slots",
    "model_timing_read", "model_timing_reset", "model_last_error",
]


class AeError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("aemodel error %d: %s" % (code, msg))
        self.code = code


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libaemodel.so is not built: run `python -m paper_2602_17681_amd.build` "
                          "(the HIP library is the only implementation; there is no fallback)")
    L = C.CDLL(_LIB_PATH)
    vp, i64p = C.c_void_p, C.POINTER(C.c_int64)
    L.model_describe.argtypes = [C.c_char_p, C.c_int, C.c_int, C.c_int, i64p, i64p, i64p, i64p, i64p]
    L.model_create.argtypes = [C.c_char_p, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    L.model_destroy.argtypes = [vp]
    L.model_destroy.restype = None
    L.model_param_count.argtypes = [vp, i64p]
    L.model_io_shape.argtypes = [vp, i64p, i64p, i64p]
    L.model_set_sample_offset.argtypes = [vp, C.c_uint64]
    L.model_forward.argtypes = [vp, vp, vp, C.c_float, C.c_uint64, vp, vp]
    L.model_backward.argtypes = [vp, vp, vp, vp, vp, vp]
    L.model_loss_mse.argtypes = [vp, vp, C.c_int64, C.c_int, vp, vp, vp]
    L.model_noise.argtypes = [C.c_uint64, C.c_uint64, C.c_int64, C.c_int64, vp, vp]
    L.model_pnorm_awgn.argtypes = [vp, vp, C.c_int64, C.c_int64, C.c_int, C.c_float, C.c_uint64, C.c_uint64, vp]
    L.model_gen_bits.argtypes = [C.c_uint64, C.c_uint64, C.c_int64, C.c_int, vp, vp]
    L.model_count_errors.argtypes = [vp, vp, C.c_int64, C.c_int, vp, vp, vp]
    L.model_monte_carlo.argtypes = [vp, vp, vp, C.c_float, C.c_uint64, C.c_uint64, C.c_uint64, vp, vp, vp, vp, vp]
    L.model_num_steps.argtypes = [vp, C.POINTER(C.c_int)]
    L.model_step_info.argtypes = [vp, C.c_int, C.POINTER(C.c_int), i64p]
    L.model_get_activation.argtypes = [vp, C.c_int, vp, vp]
    L.model_get_conv_output.argtypes = [vp, C.c_int, i64p, vp, vp]
    L.model_timing_enable.argtypes = [vp, C.c_int]
    L.model_set_overlap.argtypes = [vp, C.c_int]
    L.model_set_params_static.argtypes = [vp, C.c_int]
    L.model_set_recompute.argtypes = [vp, C.c_int]
    L.model_set_fused_backward.argtypes = [vp, C.c_int]
    L.model_set_inference.argtypes = [vp, C.c_int]
    L.model_calibrate_mfma.argtypes = [C.c_int, C.c_int, C.c_int, vp, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    L.model_mx_quantize.argtypes = [vp, vp, C.c_int64, C.c_int64, C.c_int, C.c_int, vp]
    L.model_mx_quantize_elem.argtypes = [vp, vp, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, vp]
    L.model_transform_mse_workspace.argtypes = [C.c_int64, C.c_int64, C.c_int, i64p]
    L.model_transform_mse.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int, C.c_int, vp, vp, vp, vp, vp]
    L.model_transform_mse_elem.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp]
    L.model_transform_mse_static.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp]
    L.model_inverse_shift.argtypes = [vp, vp, C.c_int64, C.c_int, vp, vp]
    L.model_lu_workspace.argtypes = [C.c_int64, C.c_int, i64p]
    L.model_lu_compose.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int, vp, vp, vp]
    L.model_lu_backward.argtypes = [vp, vp, vp, vp, vp, vp, C.c_int64, C.c_int, vp, vp, vp, vp, vp]
    L.model_vol_penalty.argtypes = [vp, C.c_int64, vp, vp, vp]
    L.model_lu_timing.argtypes = [C.c_int, C.POINTER(C.c_double), i64p]
    L.model_lu_inverse_workspace.argtypes = [C.c_int64, i64p]
    L.model_lu_inverse.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int, vp, vp, vp]
    L.model_lu_compose_batch.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int, vp, vp]
    L.model_lu_backward_batch.argtypes = [vp, vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int, vp, vp, vp, vp]
    L.model_lu_inverse_batch.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int, vp, vp]
    L.model_qr_workspace.argtypes = [C.c_int64, C.c_int, i64p]
    L.model_qr_squarings.argtypes = [vp, C.c_int64, vp, C.POINTER(C.c_int), vp]
    L.model_qr_compose.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_int, C.c_int, vp, vp, vp]
    L.model_qr_backward.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_int, C.c_int, vp, vp, vp, vp, vp]
    L.model_qr_inverse.argtypes = [vp, vp, vp, C.c_int64, C.c_int, C.c_int, vp, vp, vp, vp]
    L.model_fold_workspace.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int, i64p]
    L.model_fold_linear.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, C.c_int64, vp, vp, C.c_int64, vp, C.c_int, vp, vp, vp, vp]
    L.model_fold_embedding.argtypes = [vp, C.c_int64, C.c_int64, vp, vp, C.c_int, vp, vp]
    L.model_timing_slots.argtypes = [vp, C.POINTER(C.c_int)]
    L.model_timing_read.argtypes = [vp, C.c_int, C.c_char_p, C.c_int, C.POINTER(C.c_double), i64p,
                                    C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.model_timing_reset.argtypes = [vp]
    L.model_last_error.restype = C.c_char_p
    for name in SYMBOLS:
        if name not in ("model_destroy", "model_last_error"):
            getattr(L, name).restype = C.c_int
    return L


lib = _load()


def _check(rc):
    if rc != 0:
        raise AeError(rc, lib.model_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return C.c_void_p(t.data_ptr())


def model_last_error():
    return lib.model_last_error().decode()


def model_describe(layer_spec, batch, dtype=AE_F32, bn_mode=0):
    """Host-only: (n_params, in_chw, out_chw, latent_n, workspace_bytes)."""
    n = C.c_int64()
    lat = C.c_int64()
    ws = C.c_int64()
    ic = (C.c_int64 * 3)()
    oc = (C.c_int64 * 3)()
    _check(lib.model_describe(layer_spec.encode(), batch, dtype, bn_mode, C.byref(n), ic, oc, C.byref(lat), C.byref(ws)))
    return n.value, tuple(ic), tuple(oc), lat.value, ws.value


class Model:
    """Owns one ae_model handle (model_create / model_destroy)."""

    def __init__(self, layer_spec, batch, dtype=AE_F32, bn_mode=0):
        self._h = C.c_void_p()
        _check(lib.model_create(layer_spec.encode(), batch, dtype, bn_mode, C.byref(self._h)))
        self.batch, self.dtype, self.bn_mode, self.spec = batch, dtype, bn_mode, layer_spec
        self.tdtype = TORCH_DTYPE[dtype]
        n = C.c_int64()
        _check(lib.model_param_count(self._h, C.byref(n)))
        self.n_params = n.value
        ic = (C.c_int64 * 3)()
        oc = (C.c_int64 * 3)()
        lat = C.c_int64()
        _check(lib.model_io_shape(self._h, ic, oc, C.byref(lat)))
        self.in_shape, self.out_shape, self.latent_n = tuple(ic), tuple(oc), lat.value

    def close(self):
        if getattr(self, "_h", None) and self._h.value and lib is not None:   # lib is None at interpreter shutdown
            lib.model_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close

    def model_set_sample_offset(self, first_sample):
        _check(lib.model_set_sample_offset(self._h, first_sample))

    def model_forward(self, params, x, snr_db, seed, y):
        assert params.numel() == self.n_params and x.numel() == self.batch * _prod(self.in_shape)
        assert y.numel() == self.batch * _prod(self.out_shape)
        _check(lib.model_forward(self._h, _ptr(params, torch.float32), _ptr(x, self.tdtype), snr_db, seed,
                                 _ptr(y, self.tdtype), _stream()))

    def model_backward(self, params, x, dy, grads):
        assert params.numel() == self.n_params and grads.numel() == self.n_params
        assert dy.numel() == self.batch * _prod(self.out_shape)
        _check(lib.model_backward(self._h, _ptr(params, torch.float32), _ptr(x, self.tdtype), _ptr(dy, self.tdtype),
                                  _ptr(grads, torch.float32), _stream()))

    def model_num_steps(self):
        n = C.c_int()
        _check(lib.model_num_steps(self._h, C.byref(n)))
        return n.value

    def model_step_info(self, step):
        tok = C.c_int()
        chw = (C.c_int64 * 3)()
        _check(lib.model_step_info(self._h, step, C.byref(tok), chw))
        return tok.value, tuple(chw)

    def model_timing_enable(self, on):
        _check(lib.model_timing_enable(self._h, 1 if on else 0))

    def model_set_overlap(self, on):
        _check(lib.model_set_overlap(self._h, 1 if on else 0))

    def model_set_inference(self, on):
        _check(lib.model_set_inference(self._h, 1 if on else 0))

    def model_set_params_static(self, on):
        _check(lib.model_set_params_static(self._h, 1 if on else 0))

    def model_set_recompute(self, on):
        _check(lib.model_set_recompute(self._h, 1 if on else 0))

    def model_set_fused_backward(self, on):
        _check(lib.model_set_fused_backward(self._h, 1 if on else 0))

    def model_timing_reset(self):
        _check(lib.model_timing_reset(self._h))

    def model_timing_read(self):
        """List of dicts {name, total_ms, launches, flops, bytes} (waits for the recorded events)."""
        n = C.c_int()
        _check(lib.model_timing_slots(self._h, C.byref(n)))
        out = []
        for i in range(n.value):
            name = C.create_string_buffer(96)
            ms = C.c_double()
            cnt = C.c_int64()
            fl = C.c_double()
            by = C.c_double()
            _check(lib.model_timing_read(self._h, i, name, 96, C.byref(ms), C.byref(cnt), C.byref(fl), C.byref(by)))
            out.append(dict(name=name.value.decode(), total_ms=ms.value, launches=cnt.value, flops=fl.value,
                            bytes=by.value))
        return out

    def model_get_activation(self, step, out_nchw):
        _check(lib.model_get_activation(self._h, step, _ptr(out_nchw, torch.float32), _stream()))


    def model_get_conv_output(self, step, out_nchw=None):
        """Shape (C, H, W) of the convolution output step `step` keeps, or None if it keeps none; fills out_nchw if given."""
        chw = (C.c_int64 * 3)()
        rc = lib.model_get_conv_output(self._h, step, chw, _ptr(out_nchw, torch.float32) if out_nchw is not None else C.c_void_p(0),
                                       _stream())
        if rc == -1 and out_nchw is None:
            return None
        _check(rc)
        return tuple(chw)


def _prod(s):
    p = 1
    for v in s:
        p *= int(v)
    return p


def model_loss_mse(y, target, loss_dev, dy=None):
    dtype = AE_BF16 if y.dtype == torch.bfloat16 else AE_F32
    assert target.dtype == y.dtype and target.numel() == y.numel()
    _check(lib.model_loss_mse(_ptr(y), _ptr(target), y.numel(), dtype, _ptr(loss_dev, torch.float32),
                              _ptr(dy, y.dtype) if dy is not None else C.c_void_p(0), _stream()))


def model_noise(seed, first_sample, batch, n, out):
    assert out.numel() == batch * n
    _check(lib.model_noise(seed, first_sample, batch, n, _ptr(out, torch.float32), _stream()))


def model_pnorm_awgn(z, y, batch, n, snr_db, seed, first_sample):
    dtype = AE_BF16 if z.dtype == torch.bfloat16 else AE_F32
    assert z.numel() == batch * n and y.numel() == batch * n and y.dtype == z.dtype
    _check(lib.model_pnorm_awgn(_ptr(z), _ptr(y), batch, n, dtype, snr_db, seed, first_sample, _stream()))


def model_mx_quantize(x, q, rows, d, block=32):
    dtype = AE_BF16 if x.dtype == torch.bfloat16 else AE_F32
    assert x.numel() == rows * d and q.numel() == rows * d and q.dtype == x.dtype
    _check(lib.model_mx_quantize(_ptr(x), _ptr(q), rows, d, block, dtype, _stream()))


MX_ELEMS = {"fp4": 0, "int4": 1, "fp8": 2}


def model_mx_quantize_elem(x, q, rows, d, block, elem):
    dtype = AE_BF16 if x.dtype == torch.bfloat16 else AE_F32
    assert x.numel() == rows * d and q.numel() == rows * d and q.dtype == x.dtype
    _check(lib.model_mx_quantize_elem(_ptr(x), _ptr(q), rows, d, block, MX_ELEMS[elem] if isinstance(elem, str) else elem, dtype, _stream()))


def model_transform_mse_workspace(rows, d, dtype):
    n = C.c_int64()
    _check(lib.model_transform_mse_workspace(rows, d, dtype, C.byref(n)))
    return n.value


def model_transform_mse(x, a_mat, v, a_inv, inv_shift, rows, d, block, yq, workspace, e_blocks, e_total, elem=None):
    dtype = AE_BF16 if x.dtype == torch.bfloat16 else AE_F32
    assert x.numel() == rows * d and yq.numel() == rows * d and a_mat.numel() == d * d and a_inv.numel() == d * d
    assert a_mat.dtype == x.dtype and a_inv.dtype == x.dtype and yq.dtype == x.dtype
    assert v.numel() == d and inv_shift.numel() == d and e_blocks.numel() == d // block and e_total.numel() == 1
    assert workspace.numel() * workspace.element_size() >= model_transform_mse_workspace(rows, d, dtype)
    if elem is not None:
        _check(lib.model_transform_mse_elem(_ptr(x), _ptr(a_mat), _ptr(v, torch.float32), _ptr(a_inv), _ptr(inv_shift, torch.float32),
                                            rows, d, block, MX_ELEMS[elem], dtype, _ptr(yq), _ptr(workspace),
                                            _ptr(e_blocks, torch.float32), _ptr(e_total, torch.float32), _stream()))
        return
    _check(lib.model_transform_mse(_ptr(x), _ptr(a_mat), _ptr(v, torch.float32), _ptr(a_inv), _ptr(inv_shift, torch.float32),
                                   rows, d, block, dtype, _ptr(yq), _ptr(workspace), _ptr(e_blocks, torch.float32),
                                   _ptr(e_total, torch.float32), _stream()))


def model_inverse_shift(a_inv, v, d, inv_shift):
    dtype = AE_BF16 if a_inv.dtype == torch.bfloat16 else AE_F32
    assert a_inv.numel() == d * d and v.numel() == d and inv_shift.numel() == d
    _check(lib.model_inverse_shift(_ptr(a_inv), _ptr(v, torch.float32), d, dtype, _ptr(inv_shift, torch.float32), _stream()))


def model_transform_mse_static(x, a_mat, v, a_inv, inv_shift, rows, d, block, yq, e_blocks, e_total, elem="fp4"):
    dtype = AE_BF16 if x.dtype == torch.bfloat16 else AE_F32
    assert x.numel() == rows * d and yq.numel() == rows * d and a_mat.numel() == d * d and a_inv.numel() == d * d
    assert a_mat.dtype == x.dtype and a_inv.dtype == x.dtype and yq.dtype == x.dtype
    assert v.numel() == d and inv_shift.numel() == d and e_blocks.numel() == d // block and e_total.numel() == 1
    _check(lib.model_transform_mse_static(_ptr(x), _ptr(a_mat), _ptr(v, torch.float32), _ptr(a_inv), _ptr(inv_shift, torch.float32),
                                          rows, d, block, MX_ELEMS[elem], dtype, _ptr(yq), _ptr(e_blocks, torch.float32),
                                          _ptr(e_total, torch.float32), _stream()))


def model_lu_workspace(d, dtype):
    n = C.c_int64()
    _check(lib.model_lu_workspace(d, dtype, C.byref(n)))
    return n.value


def _lu_params(lp, up, log_s, sign_s, perm, d):
    assert lp.numel() == d * d and up.numel() == d * d and log_s.numel() == d and sign_s.numel() == d and perm.numel() == d
    return (_ptr(lp, torch.float32), _ptr(up, torch.float32), _ptr(log_s, torch.float32), _ptr(sign_s, torch.float32),
            _ptr(perm, torch.int32))


def model_lu_compose(lp, up, log_s, sign_s, perm, d, a_out, workspace):
    dtype = AE_BF16 if a_out.dtype == torch.bfloat16 else AE_F32
    assert a_out.numel() == d * d and workspace.numel() * workspace.element_size() >= model_lu_workspace(d, dtype)
    _check(lib.model_lu_compose(*_lu_params(lp, up, log_s, sign_s, perm, d), d, dtype, _ptr(a_out), _ptr(workspace), _stream()))


def model_lu_backward(g, lp, up, log_s, sign_s, perm, d, d_lp, d_up, d_log_s, workspace):
    dtype = AE_BF16 if g.dtype == torch.bfloat16 else AE_F32
    assert g.numel() == d * d and d_lp.numel() == d * d and d_up.numel() == d * d and d_log_s.numel() == d
    assert workspace.numel() * workspace.element_size() >= model_lu_workspace(d, dtype)
    _check(lib.model_lu_backward(_ptr(g), *_lu_params(lp, up, log_s, sign_s, perm, d), d, dtype, _ptr(d_lp, torch.float32),
                                 _ptr(d_up, torch.float32), _ptr(d_log_s, torch.float32), _ptr(workspace), _stream()))


def model_lu_inverse_workspace(d):
    n = C.c_int64()
    _check(lib.model_lu_inverse_workspace(d, C.byref(n)))
    return n.value


def model_lu_inverse(lp, up, log_s, sign_s, perm, d, a_inv_out, workspace):
    dtype = AE_BF16 if a_inv_out.dtype == torch.bfloat16 else AE_F32
    assert a_inv_out.numel() == d * d and workspace.numel() * workspace.element_size() >= model_lu_inverse_workspace(d)
    _check(lib.model_lu_inverse(*_lu_params(lp, up, log_s, sign_s, perm, d), d, dtype, _ptr(a_inv_out), _ptr(workspace), _stream()))


def _lu_batch_params(lp, up, log_s, sign_s, perm, count, d):
    assert lp.numel() == count * d * d and up.numel() == count * d * d
    assert log_s.numel() == count * d and sign_s.numel() == count * d and perm.numel() == count * d
    return (_ptr(lp, torch.float32), _ptr(up, torch.float32), _ptr(log_s, torch.float32), _ptr(sign_s, torch.float32),
            _ptr(perm, torch.int32))


def model_lu_compose_batch(lp, up, log_s, sign_s, perm, count, d, a_out):
    dtype = AE_BF16 if a_out.dtype == torch.bfloat16 else AE_F32
    assert a_out.numel() == count * d * d
    _check(lib.model_lu_compose_batch(*_lu_batch_params(lp, up, log_s, sign_s, perm, count, d), count, d, dtype, _ptr(a_out), _stream()))


def model_lu_backward_batch(g, lp, up, log_s, sign_s, perm, count, d, d_lp, d_up, d_log_s):
    dtype = AE_BF16 if g.dtype == torch.bfloat16 else AE_F32
    assert g.numel() == count * d * d and d_lp.numel() == count * d * d and d_up.numel() == count * d * d and d_log_s.numel() == count * d
    _check(lib.model_lu_backward_batch(_ptr(g), *_lu_batch_params(lp, up, log_s, sign_s, perm, count, d), count, d, dtype,
                                       _ptr(d_lp, torch.float32), _ptr(d_up, torch.float32), _ptr(d_log_s, torch.float32), _stream()))


def model_lu_inverse_batch(lp, up, log_s, sign_s, perm, count, d, a_inv_out):
    dtype = AE_BF16 if a_inv_out.dtype == torch.bfloat16 else AE_F32
    assert a_inv_out.numel() == count * d * d
    _check(lib.model_lu_inverse_batch(*_lu_batch_params(lp, up, log_s, sign_s, perm, count, d), count, d, dtype, _ptr(a_inv_out), _stream()))


def model_vol_penalty(log_s, d, value, d_log_s=None):
    assert log_s.numel() == d and value.numel() == 1 and (d_log_s is None or d_log_s.numel() == d)
    _check(lib.model_vol_penalty(_ptr(log_s, torch.float32), d, _ptr(value, torch.float32),
                                 _ptr(d_log_s, torch.float32) if d_log_s is not None else _ptr(None), _stream()))


def model_lu_timing(enable):
    """(milliseconds, launches) of the matrix-core products since the last call; then timing on / off."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(lib.model_lu_timing(1 if enable else 0, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def model_qr_workspace(d, squarings=5):
    n = C.c_int64()
    _check(lib.model_qr_workspace(d, squarings, C.byref(n)))
    return n.value


def model_qr_squarings(g, d, workspace):
    """The number of squarings the generator needs (synchronous: reads one float back)."""
    assert g.numel() == d * d and workspace.numel() * workspace.element_size() >= model_qr_workspace(d, 0)
    j = C.c_int(-1)
    _check(lib.model_qr_squarings(_ptr(g, torch.float32), d, _ptr(workspace), C.byref(j), _stream()))
    return j.value


def model_qr_compose(g, rp, log_s, sign_s, d, a_out, workspace, squarings=5):
    dtype = AE_BF16 if a_out.dtype == torch.bfloat16 else AE_F32
    assert g.numel() == d * d and rp.numel() == d * d and log_s.numel() == d and sign_s.numel() == d and a_out.numel() == d * d
    assert workspace.numel() * workspace.element_size() >= model_qr_workspace(d, squarings)
    _check(lib.model_qr_compose(_ptr(g, torch.float32), _ptr(rp, torch.float32), _ptr(log_s, torch.float32), _ptr(sign_s, torch.float32),
                                d, dtype, squarings, _ptr(a_out), _ptr(workspace), _stream()))


def model_qr_backward(g_a, rp, log_s, sign_s, d, d_g, d_rp, d_log_s, workspace, squarings=5):
    dtype = AE_BF16 if g_a.dtype == torch.bfloat16 else AE_F32
    assert g_a.numel() == d * d and rp.numel() == d * d and d_g.numel() == d * d and d_rp.numel() == d * d and d_log_s.numel() == d
    assert workspace.numel() * workspace.element_size() >= model_qr_workspace(d, squarings)
    _check(lib.model_qr_backward(_ptr(g_a), _ptr(rp, torch.float32), _ptr(log_s, torch.float32), _ptr(sign_s, torch.float32), d, dtype,
                                 squarings, _ptr(d_g, torch.float32), _ptr(d_rp, torch.float32), _ptr(d_log_s, torch.float32),
                                 _ptr(workspace), _stream()))


def model_qr_inverse(rp, log_s, sign_s, d, qr_workspace, a_inv_out, workspace, squarings=5):
    dtype = AE_BF16 if a_inv_out.dtype == torch.bfloat16 else AE_F32
    assert rp.numel() == d * d and a_inv_out.numel() == d * d
    assert qr_workspace.numel() * qr_workspace.element_size() >= model_qr_workspace(d, squarings)
    assert workspace.numel() * workspace.element_size() >= model_lu_inverse_workspace(d)
    _check(lib.model_qr_inverse(_ptr(rp, torch.float32), _ptr(log_s, torch.float32), _ptr(sign_s, torch.float32), d, dtype, squarings,
                                _ptr(qr_workspace), _ptr(a_inv_out), _ptr(workspace), _stream()))


def model_fold_workspace(out, in_, p, q, dtype):
    n = C.c_int64()
    _check(lib.model_fold_workspace(out, in_, p, q, dtype, C.byref(n)))
    return n.value


def model_fold_linear(w, b, out, in_, a_left, v_left, a_right_inv, v_right, w_out, b_out, workspace):
    dtype = AE_BF16 if w.dtype == torch.bfloat16 else AE_F32
    assert w.numel() == out * in_ and w_out.numel() == out * in_ and w_out.dtype == w.dtype and b_out.numel() == out
    p = 0 if a_left is None else int(round(a_left.numel() ** 0.5))
    q = 0 if a_right_inv is None else int(round(a_right_inv.numel() ** 0.5))
    assert (a_left is None or (a_left.numel() == p * p and a_left.dtype == w.dtype)) and (v_left is None or v_left.numel() == p)
    assert (a_right_inv is None or (a_right_inv.numel() == q * q and a_right_inv.dtype == w.dtype)) and (v_right is None or v_right.numel() == q)
    assert b is None or b.numel() == out
    assert workspace.numel() * workspace.element_size() >= model_fold_workspace(out, in_, p, q, dtype)
    f32 = lambda t: _ptr(None) if t is None else _ptr(t, torch.float32)
    _check(lib.model_fold_linear(_ptr(w), f32(b), out, in_, _ptr(a_left), p, f32(v_left), _ptr(a_right_inv), q, f32(v_right),
                                 dtype, _ptr(w_out), _ptr(b_out, torch.float32), _ptr(workspace), _stream()))


def model_fold_embedding(e, vocab, d, a, v, e_out):
    dtype = AE_BF16 if e.dtype == torch.bfloat16 else AE_F32
    assert e.numel() == vocab * d and e_out.numel() == vocab * d and a.numel() == d * d and a.dtype == e.dtype and e_out.dtype == e.dtype
    assert v is None or v.numel() == d
    _check(lib.model_fold_embedding(_ptr(e), vocab, d, _ptr(a), _ptr(None) if v is None else _ptr(v, torch.float32), dtype,
                                    _ptr(e_out), _stream()))


def model_calibrate_mfma(lds_reads, random_data=0, iters=4000):
    """(TFLOP/s, shader clock in MHz) of the plain matrix-core loop."""
    scratch = torch.zeros(512, dtype=torch.float32, device="cuda")
    out, mhz = C.c_double(0.0), C.c_double(0.0)
    _check(lib.model_calibrate_mfma(lds_reads, random_data, iters, _ptr(scratch), C.byref(out), C.byref(mhz), _stream()))
    return out.value, mhz.value


def model_monte_carlo(m, m_tail, params, snr_db, seed, first_sample, total_samples, x_buf, y_buf, bit_err, blk_err):
    k = m.in_shape[0]
    assert x_buf.numel() >= m.batch * k and y_buf.numel() >= m.batch * k and params.numel() == m.n_params
    assert bit_err.dtype == torch.int64 and blk_err.dtype == torch.int64
    _check(lib.model_monte_carlo(m._h, m_tail._h if m_tail is not None else C.c_void_p(0), _ptr(params, torch.float32), snr_db,
                                 seed, first_sample, total_samples, _ptr(x_buf, torch.float32), _ptr(y_buf, torch.float32),
                                 _ptr(bit_err), _ptr(blk_err), _stream()))


def model_gen_bits(seed, first_sample, batch, k, x_pm1):
    assert x_pm1.numel() == batch * k
    _check(lib.model_gen_bits(seed, first_sample, batch, k, _ptr(x_pm1, torch.float32), _stream()))


def model_count_errors(y, x_pm1, batch, k, bit_err, blk_err):
    assert y.numel() == batch * k and x_pm1.numel() == batch * k
    assert bit_err.dtype == torch.int64 and blk_err.dtype == torch.int64
    _check(lib.model_count_errors(_ptr(y, torch.float32), _ptr(x_pm1, torch.float32), batch, k, _ptr(bit_err),
                                  _ptr(blk_err), _stream()))
