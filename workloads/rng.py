"""Seeded synthetic tensor generator.

A counter-based generator: value i of stream (seed, tensor) depends only on
(seed, tensor, i), so any slice of a tensor can be produced without the rest.
64-bit counters are scrambled with the splitmix64 finaliser, mapped to
uniforms in (0, 1), and turned into normals with the Box-Muller transform in
fp64.  The result is rounded once to the tensor's storage dtype.

This module holds no arithmetic of the fused-subgraph method itself: it only
makes inputs, which both the CPU oracle and the HIP library consume as bits.
"""
import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(z):
    """splitmix64 output function on a uint64 array (wraps modulo 2**64)."""
    z = (z + np.uint64(0x9E3779B97F4A7C15)) & _MASK
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
    return z ^ (z >> np.uint64(31))


def _stream_key(seed, tensor):
    k = _mix64(np.array([seed], dtype=np.uint64))
    k = _mix64(k ^ np.array([tensor], dtype=np.uint64) * np.uint64(0xD6E8FEB86659FD93))
    return k[0]


def uniform01(seed, tensor, start, count):
    """count uniforms in (0,1), elements [start, start+count) of the stream."""
    with np.errstate(over="ignore"):
        key = _stream_key(seed, tensor)
        ctr = np.arange(start, start + count, dtype=np.uint64)
        bits = _mix64(key + ctr * np.uint64(0x2545F4914F6CDD1D))
    # 53 random bits, centred so that 0 and 1 are never produced
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed, tensor, n, mean=0.0, std=1.0, chunk=1 << 18):
    """n draws of N(mean, std) in fp64 (std is the standard deviation).

    Uniforms 2j and 2j+1 of the stream give elements 2j (cosine branch) and
    2j+1 (sine branch) of the output.
    """
    out = np.empty(n, dtype=np.float64)
    for s in range(0, n, chunk):            # chunk is even
        c = min(chunk, n - s)
        out[s:s + c] = _normal_range(seed, tensor, s, c, mean, std)
    return out


def randint(seed, tensor, index, lo, hi):
    """One integer in [lo, hi) from element `index` of the stream (host logic)."""
    u = uniform01(seed, tensor, index, 1)[0]
    return lo + min(int(u * (hi - lo)), hi - lo - 1)


# ---- storage dtypes -------------------------------------------------------
# fp32 tensors are numpy float32 arrays; bf16 tensors are numpy uint16 arrays
# holding the upper 16 bits of the fp32 pattern; fp16 tensors are numpy uint16
# arrays holding IEEE binary16 patterns.

def round_to_f32(x64):
    return x64.astype(np.float32)


def round_to_bf16_bits(x64):
    """fp64 -> fp32 -> bf16, round-to-nearest-even at each step; uint16 bits."""
    u = x64.astype(np.float32).view(np.uint32)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    r[nan] = np.uint16(0x7FC0)
    return r


def round_to_f16_bits(x64):
    """fp64 -> IEEE binary16 in one round-to-nearest-even step; uint16 bits.

    binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits; normal range 2^-14 ... 65504,
    subnormals are multiples of 2^-24; anything that rounds to 2^16 or more becomes infinity.
    """
    x = np.asarray(x64, dtype=np.float64)
    a = np.abs(x)
    with np.errstate(all="ignore"):
        _, k = np.frexp(a)                                   # a = f * 2^k, f in [0.5, 1)
        e = np.maximum(k.astype(np.int64) - 1, -14)          # subnormals share the exponent of 2^-14
        q = np.rint(np.ldexp(a, (10 - e).astype(np.int32)))  # significand in units of 2^(e-10); rint rounds half to even
        bits = (e + 14) * 1024 + q                           # the hidden bit of q supplies the +1 of the exponent field
    bits = np.where(np.isfinite(a), np.minimum(bits, 0x7C00), 0x7C00)      # overflow and infinity
    bits = np.where(a == 0, 0, bits)
    bits = np.where(np.isnan(x), 0x7E00, bits).astype(np.uint16)
    return (bits | (np.signbit(x).astype(np.uint16) << np.uint16(15))).astype(np.uint16)


def normal_stored(seed, tensor, n, dtype, mean=0.0, std=1.0, chunk=1 << 18):
    """normal() rounded to a storage dtype, made chunk by chunk to bound memory."""
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        # chunk starts are even, so the pairing of uniforms is that of normal()
        out[s:s + c] = store(_normal_range(seed, tensor, s, c, mean, std), dtype)
    return out


def _normal_range(seed, tensor, start, count, mean, std):
    """Elements [start, start+count) of normal(); start must be even."""
    m = count + (count & 1)
    u = uniform01(seed, tensor, start, m)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    ang = 2.0 * np.pi * u[1::2]
    out = np.empty(m, dtype=np.float64)
    out[0::2] = r * np.cos(ang)
    out[1::2] = r * np.sin(ang)
    out = out[:count]
    out *= std
    out += mean
    return out


def store(x64, dtype):
    """Round an fp64 array once to the named storage dtype ('f32' | 'bf16' | 'f16')."""
    if dtype == "f32":
        return round_to_f32(x64)
    if dtype == "bf16":
        return round_to_bf16_bits(x64)
    if dtype == "f16":
        return round_to_f16_bits(x64)
    raise ValueError(dtype)
