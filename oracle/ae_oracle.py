"""ctypes binding of the CPU oracle (test infrastructure, not part of the product path).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this module.
It loads oracle/libae_oracle.so, building it with g++ when it is missing.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ae_oracle.cpp")
_LIB = os.path.join(_HERE, "libae_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with the host compiler (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u32p, f32p, f64p, u64p, i64p = (C.POINTER(t) for t in (C.c_uint32, C.c_float, C.c_double, C.c_uint64, C.c_int64))
        L.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.oracle_gauss_pair.argtypes = [C.c_uint32, C.c_uint32, f32p]
        L.oracle_gauss_pair_f64.argtypes = [C.c_uint32, C.c_uint32, f64p]
        L.oracle_gauss_many.argtypes = [u32p, C.c_int64, f32p, f64p]
        L.oracle_noise.argtypes = [C.c_uint64, C.c_uint64, C.c_int64, C.c_int64, f32p]
        L.oracle_sigma.argtypes = [C.c_float]
        L.oracle_sigma.restype = C.c_float
        L.oracle_gen_bits.argtypes = [C.c_uint64, C.c_uint64, C.c_int64, C.c_int, f32p]
        L.oracle_count_errors.argtypes = [f64p, f32p, C.c_int64, C.c_int, u64p, u64p]
        L.oracle_create.argtypes = [C.c_char_p, C.c_int, C.c_int, C.c_int]
        L.oracle_create.restype = C.c_void_p
        L.oracle_destroy.argtypes = [C.c_void_p]
        L.oracle_param_count.argtypes = [C.c_void_p]
        L.oracle_param_count.restype = C.c_int64
        L.oracle_num_ops.argtypes = [C.c_void_p]
        L.oracle_op_info.argtypes = [C.c_void_p, C.c_int, i64p, i64p]
        L.oracle_forward.argtypes = [C.c_void_p, f32p, f32p, C.c_float, C.c_uint64, C.c_uint64, f64p]
        L.oracle_get_activation.argtypes = [C.c_void_p, C.c_int, f64p]
        L.oracle_get_activation.restype = C.c_int64
        L.oracle_backward.argtypes = [C.c_void_p, f32p, f64p, f64p, f64p]
        L.oracle_set_decisions.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_uint8), C.c_int64]
        L.oracle_loss_mse.argtypes = [f64p, f64p, C.c_int64, f64p]
        L.oracle_loss_mse.restype = C.c_double
        L.oracle_num_threads.restype = C.c_int
        L.oracle_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(o, C.c_uint32))
    return o


def gauss_many(words, want_f64=True):
    """words: uint32[n,2] -> (float32[n,2], float64[n,2] or None)."""
    w = np.ascontiguousarray(words, dtype=np.uint32).reshape(-1, 2)
    n = w.shape[0]
    g32 = np.zeros((n, 2), dtype=np.float32)
    g64 = np.zeros((n, 2), dtype=np.float64) if want_f64 else None
    lib().oracle_gauss_many(_p(w, C.c_uint32), n, _p(g32, C.c_float), _p(g64, C.c_double) if want_f64 else None)
    return g32, g64


def noise(seed, first_sample, batch, n):
    out = np.zeros((batch, n), dtype=np.float32)
    lib().oracle_noise(seed, first_sample, batch, n, _p(out, C.c_float))
    return out


def sigma(snr_db):
    return float(lib().oracle_sigma(C.c_float(snr_db)))


def gen_bits(seed, first_sample, batch, k):
    out = np.zeros((batch, k), dtype=np.float32)
    lib().oracle_gen_bits(seed, first_sample, batch, k, _p(out, C.c_float))
    return out


def count_errors(y, x_pm1):
    y = _f64(y)
    x = _f32(x_pm1)
    b, k = x.shape
    be = C.c_uint64(0)
    ke = C.c_uint64(0)
    lib().oracle_count_errors(_p(y, C.c_double), _p(x, C.c_float), b, k, C.byref(be), C.byref(ke))
    return be.value, ke.value


def loss_mse(y, t, want_grad=True):
    y = _f64(y)
    t = _f64(t)
    dy = np.zeros_like(y) if want_grad else None
    v = lib().oracle_loss_mse(_p(y, C.c_double), _p(t, C.c_double), y.size, _p(dy, C.c_double) if want_grad else None)
    return float(v), dy


def num_threads():
    return int(lib().oracle_num_threads())


def set_num_threads(n):
    lib().oracle_set_num_threads(int(n))


OP_KINDS = ["conv", "bn", "relu", "sigmoid", "pool2", "up2", "flatten", "fc", "reshape", "pnorm", "awgn"]


class Net:
    """One parsed network; forward() keeps every activation for backward() and for the tests."""

    def __init__(self, spec, batch, bn_mode=0, store_bf16=False):
        """store_bf16=True emulates the bfloat16 storage format: every tensor that format
        stores is rounded to bfloat16 (see the comment on Net::store_bf16 in ae_oracle.cpp)."""
        self._h = lib().oracle_create(spec.encode(), batch, bn_mode, 1 if store_bf16 else 0)
        if not self._h:
            raise ValueError("oracle: bad layer spec or batch: %r" % spec)
        self.batch = batch
        self.spec = spec
        self.n_params = int(lib().oracle_param_count(self._h))
        self.n_ops = int(lib().oracle_num_ops(self._h))
        self.ops = []
        for i in range(-1, self.n_ops):
            shp = (C.c_int64 * 3)()
            off = C.c_int64(0)
            kind = lib().oracle_op_info(self._h, i, shp, C.byref(off))
            self.ops.append(dict(kind=("in" if i < 0 else OP_KINDS[kind]), shape=tuple(shp), param_off=off.value))
        self.in_shape = self.ops[0]["shape"]
        self.out_shape = self.ops[-1]["shape"]

    def __del__(self):
        if getattr(self, "_h", None):
            lib().oracle_destroy(self._h)
            self._h = None

    def op_shape(self, i):
        """Output (C,H,W) of op i; i = -1 is the network input."""
        return self.ops[i + 1]["shape"]

    def forward(self, params, x, snr_db=10.0, seed=0, first_sample=0):
        p = _f32(params)
        assert p.size == self.n_params, (p.size, self.n_params)
        xx = _f32(x)
        assert xx.size == self.batch * int(np.prod(self.in_shape))
        y = np.zeros((self.batch,) + self.out_shape, dtype=np.float64)
        lib().oracle_forward(self._h, _p(p, C.c_float), _p(xx, C.c_float), C.c_float(snr_db), seed, first_sample,
                             _p(y, C.c_double))
        return y

    def activation(self, i):
        n = lib().oracle_get_activation(self._h, i, None)
        if n < 0:
            raise RuntimeError("oracle: forward has not run")
        out = np.zeros((self.batch,) + self.op_shape(i), dtype=np.float64)
        assert out.size == n
        lib().oracle_get_activation(self._h, i, _p(out, C.c_double))
        return out

    def set_decisions(self, i, data):
        """State the discrete decisions of op i for the following backward() calls (relu: uint8 pass bits, pool2:
        uint8 winner indices 0..3, shape of the op's output); data=None withdraws them."""
        if data is None:
            rc = lib().oracle_set_decisions(self._h, i, None, 0)
        else:
            d = np.ascontiguousarray(data, dtype=np.uint8)
            rc = lib().oracle_set_decisions(self._h, i, _p(d, C.c_uint8), d.size)
        if rc != 0:
            raise ValueError("oracle: op %d takes no decisions of that size" % i)

    def backward(self, params, dy):
        p = _f32(params)
        g = _f64(dy)
        grads = np.zeros(self.n_params, dtype=np.float64)
        dx = np.zeros((self.batch,) + self.in_shape, dtype=np.float64)
        rc = lib().oracle_backward(self._h, _p(p, C.c_float), _p(g, C.c_double), _p(grads, C.c_double), _p(dx, C.c_double))
        if rc != 0:
            raise RuntimeError("oracle: backward before forward")
        return grads, dx
