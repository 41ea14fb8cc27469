"""Seeded synthetic tensors for the CNN workloads (stand-ins for the paper's
datasets and trained weights, Table 4 of arXiv 2109.01611).

This module serves both the CPU oracle and the HIP path and therefore holds
none of the method's arithmetic: it only draws numbers.  The generator is
counter based, so element ``i`` of tensor ``name`` under ``seed`` is a pure
function of ``(seed, name, i)`` and does not depend on any library's stream:

* 64-bit words come from the SplitMix64 output function (Steele, Lea, Flood,
  "Fast splittable pseudorandom number generators", OOPSLA 2014) applied to
  ``key + (i + 1) * golden_gamma`` where ``key`` mixes the seed with an
  FNV-1a hash of the tensor name;
* uniforms are the top 53 bits, offset by half an ulp so 0 is never drawn;
* normals are Box-Muller over two words per element.

Every tensor is returned as float32 whose values are exactly representable
in bfloat16 (rounded to nearest even), so both sides start from identical
numbers; biases stay plain float32.
"""

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _fnv1a64(text):
    h = 0xCBF29CE484222325
    for byte in text.encode("utf-8"):
        h ^= byte
        h = (h * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed, name):
    k = np.array([(int(seed) * 0xD1342543DE82EF95 + _fnv1a64(name)) & 0xFFFFFFFFFFFFFFFF],
                 dtype=np.uint64)
    return _mix(k)[0]


def words(seed, name, start, count):
    """``count`` 64-bit words of stream ``(seed, name)`` from counter ``start``."""
    idx = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(_key(seed, name) + idx * _GAMMA)


def _unit(w):
    return ((w >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform(seed, name, n):
    """``n`` float64 draws from U(0, 1)."""
    out = np.empty(n, dtype=np.float64)
    for lo in range(0, n, _CHUNK):
        m = min(_CHUNK, n - lo)
        out[lo:lo + m] = _unit(words(seed, name, lo, m))
    return out


def normal(seed, name, n):
    """``n`` float64 draws from N(0, 1) (Box-Muller, two words per element)."""
    out = np.empty(n, dtype=np.float64)
    for lo in range(0, n, _CHUNK):
        m = min(_CHUNK, n - lo)
        w = words(seed, name, 2 * lo, 2 * m)
        u1 = _unit(w[0::2])
        u2 = _unit(w[1::2])
        out[lo:lo + m] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return out


def bf16_bits(a):
    """float32 array -> uint16 bfloat16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits):
    """uint16 bfloat16 bit patterns -> float32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a):
    """float array -> float32 holding the nearest bfloat16 values."""
    a32 = np.asarray(a, dtype=np.float32)
    return bf16_to_f32(bf16_bits(a32)).reshape(a32.shape)


def tensor(seed, name, shape, dist, scale=1.0, quantise=True):
    """Seeded tensor: ``dist`` is ``"normal"`` (N(0, scale^2)) or ``"uniform"``
    (U(0, scale)).  ``quantise`` rounds to bfloat16-representable float32."""
    n = int(np.prod(shape, dtype=np.int64))
    if dist == "normal":
        v = normal(seed, name, n)
    elif dist == "uniform":
        v = uniform(seed, name, n)
    else:
        raise ValueError("unknown distribution %r" % (dist,))
    v = (v * scale).astype(np.float32).reshape(shape)
    return bf16_round(v) if quantise else v


def he_normal(seed, name, shape):
    """He-normal weights N(0, 2 / fan_in); ``shape`` is (K, C, R, S) for a
    convolution or (Out, In) for a fully connected layer."""
    fan_in = int(np.prod(shape[1:], dtype=np.int64))
    return tensor(seed, name, shape, "normal", scale=float(np.sqrt(2.0 / fan_in)))


def bias(seed, name, n):
    """Bias vector N(0, 0.1^2), float32 (not quantised)."""
    return tensor(seed, name, (n,), "normal", scale=0.1, quantise=False)
