"""Workload descriptions and seeded synthetic input generators.

This module is shared by the tests, the benchmark and the smoke check, and feeds
both the GPU library and the CPU oracle.  It holds NO arithmetic of the method:
only the five benchmark network descriptions (as layer-spec strings), a walker that
turns a spec into the shapes / offsets of the parameter blob, and random-number
recipes for inputs and initial parameters.
"""
import numpy as np


def _enc(chs):
    return ",".join("conv3:%d,bn,relu,pool2" % c for c in chs)


def _dec(chs):
    parts = ["up2,conv3:%d,relu" % c for c in chs[:-1]]
    parts.append("up2,conv3:%d,sigmoid" % chs[-1])
    return ",".join(parts)


# The five benchmark configurations (batch, storage dtype, seed, SNR points, whether
# the configuration trains).  Decoder composition: the decoder fc / 1x1 conv has no
# activation, every up2+conv3 is followed by ReLU and the last by sigmoid, no
# batch-norm in the decoder (the tiny configuration spells this out; the others
# mirror the encoder's channel list in reverse).
CONFIGS = {
    "cfg1": dict(
        spec="in:1x28x28," + _enc([16, 32]) + ",flatten,fc:64,pnorm,awgn,fc:1568,reshape:32x7x7," + _dec([16, 1]),
        batch=64, dtype="f32", seed=0, snr_db=[10.0], backward=False),
    "cfg2": dict(
        spec="in:3x32x32," + _enc([64, 128, 256]) + ",flatten,fc:512,pnorm,awgn,fc:4096,reshape:256x4x4," + _dec([128, 64, 3]),
        batch=256, dtype="f32", seed=1, snr_db=[0.0, 5.0, 10.0, 20.0], backward=True),
    "cfg3": dict(
        spec="in:3x64x64," + _enc([128, 256, 512]) + ",flatten,fc:1024,pnorm,awgn,fc:32768,reshape:512x8x8," + _dec([256, 128, 3]),
        batch=128, dtype="bf16", seed=2, snr_db=[5.0], backward=True),
    "cfg4": dict(
        spec="in:64x1x1,fc:512,relu,fc:512,relu,fc:128,pnorm,awgn,fc:512,relu,fc:512,relu,fc:64,sigmoid",
        batch=65536, dtype="f32", seed=3, snr_db=[-2.0, 0.0, 2.0, 4.0], backward=False, total_samples=100_000_000),
    "cfg5": dict(
        spec="in:3x256x256," + _enc([64, 128, 256, 512, 512]) + ",conv1:64,pnorm,awgn,conv1:512," + _dec([512, 256, 128, 64, 3]),
        batch=32, dtype="bf16", seed=4, snr_db=[10.0], backward=True),
}


def scaled_spec(name, hw):
    """The same network as CONFIGS[name] on a smaller square input (conv configs only);
    the fc widths that depend on the spatial size are recomputed."""
    cfg = CONFIGS[name]
    toks = cfg["spec"].split(",")
    c0 = int(toks[0][3:].split("x")[0])
    n_pool = sum(t == "pool2" for t in toks)
    assert hw % (1 << n_pool) == 0
    out = ["in:%dx%dx%d" % (c0, hw, hw)]
    small = hw >> n_pool
    for i, t in enumerate(toks[1:], 1):
        if t.startswith("reshape:"):
            c = int(t[8:].split("x")[0])
            out.append("reshape:%dx%dx%d" % (c, small, small))
        elif t.startswith("fc:") and i + 1 < len(toks) and toks[i + 1].startswith("reshape:"):
            c = int(toks[i + 1][8:].split("x")[0])
            out.append("fc:%d" % (c * small * small))
        else:
            out.append(t)
    return ",".join(out)


def param_layout(spec, bn_mode=0):
    """Walk a layer spec; return (entries, n_params, in_shape, out_shape).
    entries: dicts {op, name, kind ('w','b','gamma','beta','rmean','rvar'), shape, offset, fan_in}
    in blob order: conv W[co][ci][k][k], b[co]; fc W[out][in], b[out]; bn gamma, beta
    (+ running mean, var when bn_mode = 1)."""
    toks = [t.strip() for t in spec.split(",")]
    assert toks[0].startswith("in:")
    c, h, w = (int(v) for v in toks[0][3:].split("x"))
    in_shape = (c, h, w)
    off = 0
    ent = []

    def add(op, name, kind, shape, fan_in=0):
        nonlocal off
        ent.append(dict(op=op, name=name, kind=kind, shape=tuple(shape), offset=off, fan_in=fan_in))
        off += int(np.prod(shape))

    for i, t in enumerate(toks[1:]):
        if t.startswith("conv3:") or t.startswith("conv1:"):
            k = int(t[4])
            co = int(t[6:])
            add(i, t, "w", (co, c, k, k), c * k * k)
            add(i, t, "b", (co,))
            c = co
        elif t.startswith("fc:"):
            assert h == 1 and w == 1
            co = int(t[3:])
            add(i, t, "w", (co, c), c)
            add(i, t, "b", (co,))
            c = co
        elif t == "bn":
            add(i, t, "gamma", (c,))
            add(i, t, "beta", (c,))
            if bn_mode == 1:
                add(i, t, "rmean", (c,))
                add(i, t, "rvar", (c,))
        elif t == "pool2":
            h, w = h // 2, w // 2
        elif t == "up2":
            h, w = h * 2, w * 2
        elif t == "flatten":
            c, h, w = c * h * w, 1, 1
        elif t.startswith("reshape:"):
            c, h, w = (int(v) for v in t[8:].split("x"))
        elif t in ("relu", "sigmoid", "pnorm", "awgn"):
            pass
        else:
            raise ValueError("unknown token %r" % t)
    return ent, off, in_shape, (c, h, w)


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def f32_to_bf16_bits(a):
    """float32 values that are exactly representable in bfloat16 -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def make_params(spec, seed, bn_mode=0, perturb=False, bf16=False):
    """Initial parameter blob (float32).  Weights Kaiming-normal N(0, 2/fan_in), bias 0,
    gamma 1, beta 0 (running mean 0, running var 1).  perturb=True makes biases, gamma,
    beta (and running statistics) non-trivial so that tests exercise them.  bf16=True
    rounds every value to a bfloat16-representable float32."""
    ent, n, _, _ = param_layout(spec, bn_mode)
    rng = np.random.default_rng([seed, 0x5EED])
    p = np.zeros(n, dtype=np.float32)
    for e in ent:
        sz = int(np.prod(e["shape"]))
        sl = slice(e["offset"], e["offset"] + sz)
        if e["kind"] == "w":
            p[sl] = rng.standard_normal(sz).astype(np.float32) * np.float32(np.sqrt(2.0 / e["fan_in"]))
        elif e["kind"] == "b":
            p[sl] = 0.1 * rng.standard_normal(sz).astype(np.float32) if perturb else 0.0
        elif e["kind"] == "gamma":
            p[sl] = 1.0 + (0.2 * rng.standard_normal(sz).astype(np.float32) if perturb else 0.0)
        elif e["kind"] == "beta":
            p[sl] = 0.1 * rng.standard_normal(sz).astype(np.float32) if perturb else 0.0
        elif e["kind"] == "rmean":
            p[sl] = 0.1 * rng.standard_normal(sz).astype(np.float32) if perturb else 0.0
        elif e["kind"] == "rvar":
            p[sl] = 1.0 + (0.5 * rng.random(sz).astype(np.float32) if perturb else 0.0)
    return round_to_bf16(p) if bf16 else p


def make_input(spec, batch, seed, bf16=False):
    """Uniform [0,1) images, float32 NCHW."""
    _, _, in_shape, _ = param_layout(spec)
    rng = np.random.default_rng([seed, 0xDA7A])
    x = rng.random((batch,) + in_shape, dtype=np.float32)
    return round_to_bf16(x) if bf16 else x


def make_cotangent(shape, seed, bf16=False):
    """A generic upstream gradient for backward tests."""
    rng = np.random.default_rng([seed, 0xC07A])
    g = rng.standard_normal(shape).astype(np.float32)
    return round_to_bf16(g) if bf16 else g


def make_activations(rows, d, seed, bf16=False):
    """Synthetic stand-in for transformer activations [tokens][d] (float32): Gaussian entries with a
    log-normal scale per channel and per token and a few outlier channels two orders of magnitude
    above the rest (the heavy tails that block-wise scaling has to cope with).  No arithmetic of
    the quantiser lives here."""
    rng = np.random.default_rng([seed, 0xAC71])
    x = rng.standard_normal((rows, d), dtype=np.float32)
    chan = np.exp(rng.standard_normal(d).astype(np.float32))
    chan[rng.choice(d, size=max(1, d // 512), replace=False)] *= 100.0
    tok = np.exp(0.5 * rng.standard_normal((rows, 1)).astype(np.float32))
    x = x * chan[None, :] * tok
    return round_to_bf16(x) if bf16 else x


def make_transform(d, seed, bf16=False, kind="affine"):
    """An invertible d x d matrix A, a shift v and A^-1 for the transformation-error path (float32 arrays; the
    inverse is taken in float64 of the matrix AS STORED, then stored in the same type).  The constant term of the
    inverse map is the method's own arithmetic and is formed by each side for itself.
    kind: "identity", "hadamard" (orthonormal Walsh-Hadamard, d a power of two), "affine" (a random
    rotation times per-channel gains in [0.5, 2], plus a dense perturbation, with a shift)."""
    rng = np.random.default_rng([seed, 0x7A4F])
    if kind == "identity":
        a = np.eye(d)
        v = np.zeros(d)
    elif kind == "hadamard":
        a = np.array([[1.0]])
        while a.shape[0] < d:
            a = np.block([[a, a], [a, -a]])
        a = a / np.sqrt(d)
        v = np.zeros(d)
    else:
        q, _ = np.linalg.qr(rng.standard_normal((d, d)))
        a = q * np.exp(rng.uniform(-0.7, 0.7, size=d))[None, :] + 0.02 * rng.standard_normal((d, d)) / np.sqrt(d)
        v = 0.5 * rng.standard_normal(d)
    a = a.astype(np.float32)
    if bf16:
        a = round_to_bf16(a)
    ainv = np.linalg.inv(a.astype(np.float64)).astype(np.float32)
    if bf16:
        ainv = round_to_bf16(ainv)
    return a, v.astype(np.float32), ainv


def make_lu_params(d, seed, kind="random", noise=0.0, block=32):
    """Free parameters of the LU parametrisation A = P L (U + diag(s)): (Lp, Up, log_s, sign, perm), float32 arrays
    (perm int32; (P M)[i] = M[perm[i]]).
    kind "random": a random permutation, dense Gaussian triangles of size 1/sqrt(d), log|s| ~ N(0, 0.3), random signs.
    kind "bd_hadamard": the paper's initialisation for this parametrisation — A is block diagonal with blocks of
    `block` x `block` randomly signed orthonormal Hadamard matrices, given here by the exact factors of each block
    (partial-pivoting LU, a library routine); `noise` > 0 adds Gaussian noise of that size to the free parameters
    outside the diagonal blocks (reading: the small off-block noise of the initialisation enters through the
    parameters)."""
    rng = np.random.default_rng([seed, 0x1D5])
    if kind == "random":
        perm = rng.permutation(d).astype(np.int32)
        lp = rng.standard_normal((d, d)) / np.sqrt(d)
        up = rng.standard_normal((d, d)) / np.sqrt(d)
        log_s = 0.3 * rng.standard_normal(d)
        sign = rng.choice([-1.0, 1.0], size=d)
    else:
        import scipy.linalg
        assert d % block == 0 and block & (block - 1) == 0
        h = np.array([[1.0]])
        while h.shape[0] < block:
            h = np.block([[h, h], [h, -h]])
        h /= np.sqrt(block)
        perm = np.zeros(d, dtype=np.int32)
        lp, up = np.zeros((d, d)), np.zeros((d, d))
        log_s, sign = np.zeros(d), np.ones(d)
        for b in range(d // block):
            hb = h * rng.choice([-1.0, 1.0], size=block)[None, :]           # random column signs
            pm, l, u = scipy.linalg.lu(hb)                                   # hb = pm @ l @ u
            o = b * block
            perm[o:o + block] = o + np.argmax(pm, axis=1)                    # (pm M)[i] = M[argmax_j pm[i, j]]
            lp[o:o + block, o:o + block] = np.tril(l, -1)
            up[o:o + block, o:o + block] = np.triu(u, 1)
            log_s[o:o + block] = np.log(np.abs(np.diag(u)))
            sign[o:o + block] = np.sign(np.diag(u))
        if noise > 0.0:
            off = np.kron(np.eye(d // block), np.ones((block, block))) == 0
            lp += noise * rng.standard_normal((d, d)) * off
            up += noise * rng.standard_normal((d, d)) * off
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    return f(lp), f(up), f(log_s), f(sign), perm


def make_qr_params(d, seed, kind="random", noise=0.0, block=32):
    """Free parameters of the QR parametrisation A = exp((G - G^T)/2) (R + diag(s)): (G, Rp, log_s, sign), float32.
    kind "random": dense Gaussian G and R of size 1/sqrt(d), log|s| ~ N(0, 0.3), random signs.
    kind "bd_orthogonal": the paper's initialisation for this parametrisation — A is block diagonal with blocks of
    `block` x `block` random rotations (each block's G is the real skew-symmetric logarithm of the rotation, a
    library routine; R = 0, s = 1); `noise` > 0 adds Gaussian noise of that size to G and R outside the diagonal
    blocks."""
    rng = np.random.default_rng([seed, 0x9A7])
    if kind == "random":
        g = rng.standard_normal((d, d)) / np.sqrt(d)
        rp = rng.standard_normal((d, d)) / np.sqrt(d)
        log_s = 0.3 * rng.standard_normal(d)
        sign = rng.choice([-1.0, 1.0], size=d)
    else:
        import scipy.linalg
        assert d % block == 0
        g, rp = np.zeros((d, d)), np.zeros((d, d))
        log_s, sign = np.zeros(d), np.ones(d)
        for b in range(d // block):
            q, r = np.linalg.qr(rng.standard_normal((block, block)))
            q = q * np.sign(np.diag(r))[None, :]
            if np.linalg.det(q) < 0:
                q[:, 0] = -q[:, 0]                                   # a rotation: determinant +1, so a real logarithm exists
            lg = np.real(scipy.linalg.logm(q))
            o = b * block
            g[o:o + block, o:o + block] = 0.5 * (lg - lg.T)
        if noise > 0.0:
            off = np.kron(np.eye(d // block), np.ones((block, block))) == 0
            g += noise * rng.standard_normal((d, d)) * off
            rp += noise * rng.standard_normal((d, d)) * off
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    return f(g), f(rp), f(log_s), f(sign)
