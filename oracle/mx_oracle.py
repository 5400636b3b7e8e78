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
The integer element format mentioned in the paper ("INT4" under MX scaling) is not an OCP format
and is not built: parity unpinned.
"""
import numpy as np

E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])   # index = 3-bit magnitude code (exponent:mantissa)
E2M1_RMAX = 2
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


def block_scale_exponent(amax):
    """floor(log2(amax)) - r_max, clamped to the E8M0 range; amax > 0 (float64, exact via frexp)."""
    m, e = np.frexp(amax)                                   # amax = m * 2^e, 0.5 <= m < 1  =>  floor(log2 amax) = e - 1
    return np.clip(e - 1 - E2M1_RMAX, SCALE_EXP_MIN, SCALE_EXP_MAX)


def mx_quantize(x, block=32):
    """Q(x) of Eq. (1) for a [rows][d] array, blocks of `block` consecutive elements of a row."""
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] % block == 0
    xb = x.reshape(-1, block)
    out = np.zeros_like(xb)
    amax = np.abs(xb).max(axis=1)
    nz = amax > 0.0
    k = block_scale_exponent(amax[nz])
    s = np.ldexp(1.0, k)[:, None]
    out[nz] = s * quantize_element_e2m1(xb[nz] / s)
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
