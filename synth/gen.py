"""Seeded synthetic tensors, served identically to the CPU oracle and to the HIP path.

Counter-based: element i of a stream depends only on (seed, i), so a tensor is reproducible on
any machine and any slice of it can be regenerated. Nothing here knows about convolution.

Value recipes: uniform[lo,hi), Gaussian(0, std) via Box-Muller in fp64 cast to fp32, small
integers (for bit-exact comparisons), and round-to-nearest-even bfloat16 quantisation.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

BASE_SEED = 14126249 * 1000


def tensor_seed(config, tensor_index):
    return BASE_SEED + 100 * int(config) + int(tensor_index)


def _mix64(counter, seed):
    """splitmix64 output function applied to seed + (counter+1)*golden (wrapping)."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed) + (counter + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(n, seed, stream=0, chunk=1 << 24):
    """n doubles in [0,1) with 24-bit resolution (exactly representable in fp32)."""
    out = np.empty(n, dtype=np.float64)
    offs = np.uint64(stream) << np.uint64(40)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        ctr = np.arange(a, b, dtype=np.uint64) + offs
        out[a:b] = (_mix64(ctr, seed) >> np.uint64(40)).astype(np.float64) * (2.0 ** -24)
    return out


def uniform(shape, seed, lo=0.0, hi=1.0):
    n = int(np.prod(shape))
    return (lo + (hi - lo) * _unit(n, seed)).astype(np.float32).reshape(shape)


def gaussian(shape, seed, std=0.01):
    n = int(np.prod(shape))
    u1 = _unit(n, seed, stream=1)
    u2 = _unit(n, seed, stream=2)
    r = np.sqrt(-2.0 * np.log(1.0 - u1))  # 1-u1 in (0,1]
    z = r * np.cos(2.0 * np.pi * u2)
    return (std * z).astype(np.float32).reshape(shape)


def integers(shape, seed, amax=4):
    """Small integers in [-amax, amax] stored as fp32 (every partial sum stays exact)."""
    n = int(np.prod(shape))
    u = _unit(n, seed, stream=3)
    return (np.floor(u * (2 * amax + 1)) - amax).astype(np.float32).reshape(shape)


def to_bf16_bits(a):
    """fp32 array -> uint16 bfloat16 bit patterns, round to nearest even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b):
    """uint16 bfloat16 bit patterns -> fp32 array (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize_bf16(a):
    """fp32 array rounded to the nearest bfloat16 value, returned as fp32."""
    return from_bf16_bits(to_bf16_bits(a)).reshape(np.shape(a))


def layer_tensors(layer, config, layer_index=0, integer=False, amax=None):
    """x, w, b, dy for one conv layer, standalone.

    Recipe: x ~ uniform[0,1), w and b ~ Gaussian(0, std 0.01), dy ~ uniform[-1,1); config 1 draws
    all four from uniform[-1,1). bf16 layers are quantised to bfloat16 values (still returned as
    fp32 arrays; both sides read the same 16-bit patterns after `to_bf16_bits`).
    With integer=True all four are small integers so that any summation order is exact.
    """
    base = 10 * layer_index
    sx, sw, sb, sdy = (tensor_seed(config, base + i) for i in range(4))
    if integer:
        ax, aw = amax if amax is not None else (2, 2)
        x = integers(layer.x_shape, sx, ax)
        w = integers(layer.w_shape, sw, aw)
        b = integers((layer.K,), sb, ax)
        dy = integers(layer.y_shape, sdy, aw)
    elif config == 1:
        x = uniform(layer.x_shape, sx, -1, 1)
        w = uniform(layer.w_shape, sw, -1, 1)
        b = uniform((layer.K,), sb, -1, 1)
        dy = uniform(layer.y_shape, sdy, -1, 1)
    else:
        x = uniform(layer.x_shape, sx, 0, 1)
        w = gaussian(layer.w_shape, sw, 0.01)
        b = gaussian((layer.K,), sb, 0.01)
        dy = uniform(layer.y_shape, sdy, -1, 1)
    if layer.dtype == "bf16":
        x, w, b, dy = (quantize_bf16(t) for t in (x, w, b, dy))
    return x, w, b, dy


def fast_uniform(shape, seed, lo=0.0, hi=1.0):
    """Philox-based uniform fp32 tensor for the full-size workloads (hundreds of millions of
    elements), where the pure-numpy splitmix stream above would take minutes."""
    g = np.random.Generator(np.random.Philox(int(seed)))
    a = g.random(size=shape, dtype=np.float32)
    if lo != 0.0 or hi != 1.0:
        a *= np.float32(hi - lo)
        a += np.float32(lo)
    return a


def fast_gaussian(shape, seed, std=0.01):
    g = np.random.Generator(np.random.Philox(int(seed)))
    a = g.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    return a


def layer_tensors_fast(layer, config, layer_index=0):
    """Same recipe as layer_tensors (x~U[0,1), w,b~N(0,0.01), dy~U[-1,1)) on the fast generator."""
    base = 10 * layer_index
    sx, sw, sb, sdy = (tensor_seed(config, base + i) for i in range(4))
    x = fast_uniform(layer.x_shape, sx, 0, 1)
    w = fast_gaussian(layer.w_shape, sw, 0.01)
    b = fast_gaussian((layer.K,), sb, 0.01)
    dy = fast_uniform(layer.y_shape, sdy, -1, 1)
    if layer.dtype == "bf16":
        x, w, b, dy = (quantize_bf16(t) for t in (x, w, b, dy))
    return x, w, b, dy
