"""CPU oracle of the MX block quantiser Q(x) (test infrastructure, not part of the product path).

Follows the paper's Section "MX quantization", Eq. (1): per block of B consecutive elements of a
row, the scale is the power of two  s = 2^(floor(log2(max_j |x_j|)) - r_max)  and every element
becomes  s * Q_e(x_j / s),  with Q_e the element quantiser of the low-precision format and r_max
the largest exponent of that format.  Only tests, the smoke check and the benchmark's
cpu_baseline leg import this module; it shares no code with the HIP path.

Element format: FP4 E2M1 (the OCP microscaling element format the paper's experiments use with
B = 32): magnitudes {0, 0.5, 1, 1.5, 2, 3, 4, 6}, r_max = 2 (6 = 1.5 * 2^2).

Readings where the paper is silent (each one is listed in the design document):
  * Q_e rounds to the NEAREST representable value, ties to the value whose code has an even
    mantissa bit (round-to-nearest-even, as in the OCP specification's conversions), and
    saturates at +-6 (a scaled block maximum lies in [4, 8), so (6, 8) clips);
  * an all-zero block quantises to zeros (its scale is undefined);
  * the scale exponent is clamped to the E8M0 range [-127, 127];
  * plain numpy in float64, one obviously-correct nearest-value search per element: no blocking
    tricks, no bit manipulation.
Other element formats (`fmt` argument of mx_quantize / quantize_element):
  * "fp8": FP8 E4M3 of the OCP 8-bit floating point specification (bias 7, subnormals k * 2^-9, normals
    (1 + m/8) * 2^(e-7), no infinities, the all-ones code is NaN: largest value 448 = 1.75 * 2^8), r_max = 8;
  * "int4": the integer element format the paper evaluates under MX scaling is not an OCP format and the paper does
    not define it — PARITY UNPINNED.  Reading, by analogy with the OCP MXINT8 element (two's complement with an
    implied scale that puts the values in (-2, 2)): magnitudes k/4, k = 0..7, symmetric (the code -8 unused),
    r_max = 0, round to nearest, ties to the even integer, saturating at 1.75.
"""
import numpy as np

E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])   # index = 3-bit magnitude code (exponent:mantissa)
E2M1_RMAX = 2
# FP8 E4M3: index = 7-bit magnitude code (4 exponent bits : 3 mantissa bits), the NaN code 0x7F left out
E4M3_GRID = np.array([(m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
                      for e in range(16) for m in range(8)][:-1])
INT4_GRID = np.arange(8) / 4.0                                     # reading (unpinned): see the header
FORMATS = {"fp4": (E2M1_GRID, E2M1_RMAX), "fp8": (E4M3_GRID, 8), "int4": (INT4_GRID, 0)}
SCALE_EXP_MIN, SCALE_EXP_MAX = -127, 127


def quantize_element_e2m1(y):
    """Q_e: nearest E2M1 value of every entry of y (float64), ties to the even code, saturating."""
    y = np.asarray(y, dtype=np.float64)
    a = np.abs(y)
    dist = np.abs(a[..., None] - E2M1_GRID)                 # distance to each of the eight magnitudes
    best = dist.min(axis=-1, keepdims=True)
    cand = dist == best                                     # one candidate, or two adjacent ones on a tie
    even = cand & (np.arange(8) % 2 == 0)
    pick = np.where(even.any(axis=-1), even.argmax(axis=-1), cand.argmax(axis=-1))
    return np.sign(y) * E2M1_GRID[pick]


def quantize_element(y, fmt="fp4"):
    """Q_e of the named element format: nearest magnitude of its grid, ties to the even code, saturating."""
    if fmt == "fp4":
        return quantize_element_e2m1(y)
    grid = FORMATS[fmt][0]
    y = np.asarray(y, dtype=np.float64)
    a = np.abs(y).reshape(-1)
    out = np.empty_like(a)
    for lo in range(0, a.size, 1 << 16):                    # (bounded memory: the grid has up to 127 entries)
        dist = np.abs(a[lo:lo + (1 << 16), None] - grid)
        best = dist.min(axis=-1, keepdims=True)
        cand = dist == best
        even = cand & (np.arange(grid.size) % 2 == 0)
        pick = np.where(even.any(axis=-1), even.argmax(axis=-1), cand.argmax(axis=-1))
        out[lo:lo + (1 << 16)] = grid[pick]
    return np.sign(y) * out.reshape(y.shape)


def block_scale_exponent(amax, r_max=E2M1_RMAX):
    """floor(log2(amax)) - r_max, clamped to the E8M0 range; amax > 0 (float64, exact via frexp)."""
    m, e = np.frexp(amax)                                   # amax = m * 2^e, 0.5 <= m < 1  =>  floor(log2 amax) = e - 1
    return np.clip(e - 1 - r_max, SCALE_EXP_MIN, SCALE_EXP_MAX)


def mx_quantize(x, block=32, fmt="fp4"):
    """Q(x) of Eq. (1) for a [rows][d] array, blocks of `block` consecutive elements of a row."""
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] % block == 0
    xb = x.reshape(-1, block)
    out = np.zeros_like(xb)
    amax = np.abs(xb).max(axis=1)
    nz = amax > 0.0
    k = block_scale_exponent(amax[nz], FORMATS[fmt][1])
    s = np.ldexp(1.0, k)[:, None]
    out[nz] = s * quantize_element(xb[nz] / s, fmt)
    return out.reshape(x.shape)


def block_scales(x, block=32):
    """The scales s_i (0 for all-zero blocks), shape [rows][d / block]."""
    x = np.asarray(x, dtype=np.float64)
    xb = x.reshape(-1, block)
    amax = np.abs(xb).max(axis=1)
    s = np.zeros_like(amax)
    nz = amax > 0.0
    s[nz] = np.ldexp(1.0, block_scale_exponent(amax[nz]))
    return s.reshape(x.shape[0], -1)


# ---------------------------------------------------------------------------------------------
# Transformation mean squared error (the paper's Definition "Transformation Mean Squared Error",
# Eq. (2), and the block-wise error of its numerical analysis):
#   T(x) = A x + v,   T^-1(y) = A^-1 y - A^-1 v,
#   E(T)     = 1/d * mean over tokens of || x - T^-1(Q(T(x))) ||^2,
#   E_B^i(T) = 1/B * sum over the channels j of block i of (x - T^-1(Q(T(x))))_j^2, averaged over tokens.
# The inverse is an input (the caller supplies A^-1; nothing here inverts a matrix).
# Reading: T(x) is rounded to the tensor's storage type (bf16 or binary32) before it is
# quantised, like every stored activation; everything else is float64.
# ---------------------------------------------------------------------------------------------
def _round_bf16(a):
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a)).astype(np.float64)


def transform_mse(x, A, v, Ainv, block=32, storage="f64", fmt="fp4"):
    """Returns (E, E_blocks[d / block], yq) for tokens x [n][d]; storage in {"f64", "f32", "bf16"}."""
    x = np.asarray(x, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    Ainv = np.asarray(Ainv, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n, d = x.shape
    y = x @ A.T + v                                        # T(x), token by token
    if storage == "bf16":
        y = _round_bf16(y)
    elif storage == "f32":
        y = y.astype(np.float32).astype(np.float64)
    yq = mx_quantize(y, block, fmt)
    e, e_blocks = reconstruction_error(x, yq, v, Ainv, block)
    return e, e_blocks, yq


def reconstruction_error(x, yq, v, Ainv, block=32):
    """The second half of Eq. 2 on given quantised values yq = Q(T(x)) [n][d]: (E, E_blocks[d / block]) of
    x - T^-1(yq).  Separate so that a test can hold a device's error sums against its own quantisation decisions."""
    x = np.asarray(x, dtype=np.float64)
    yq = np.asarray(yq, dtype=np.float64)
    Ainv = np.asarray(Ainv, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n, d = x.shape
    xhat = yq @ Ainv.T - Ainv @ v                          # T^-1(Q(T(x)))
    err2 = (x - xhat) ** 2
    e_blocks = err2.reshape(n, d // block, block).sum(axis=2).mean(axis=0) / block
    return float(err2.sum() / (n * d)), e_blocks
