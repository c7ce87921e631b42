"""Seeded, counter-based synthetic inputs (no method arithmetic).

Every value is a pure function of (seed, stream name, element index), so the
CPU oracle's tests and the HIP path's tests see bit-identical inputs without
either side depending on the other.  The synthetic tensors stand in for the
CIFAR-10/100 and ImageNet mini-batches of Sec. 5 (shapes and class counts only).
"""
import zlib
import numpy as np

from .configs import NetDesc, ModuleDesc, module_tensor_specs, aux_tensor_specs

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(z: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _stream_key(seed: int, stream: str) -> np.uint64:
    h = zlib.crc32(stream.encode()) & 0xFFFFFFFF
    return np.uint64(((seed & 0xFFFFFFFF) << 32) | h)


def _u01(seed: int, stream: str, lane: int, n: int) -> np.ndarray:
    """n uniforms in (0,1): counter = 2*i + lane hashed with the stream key."""
    key = _mix(np.array([_stream_key(seed, stream)], dtype=np.uint64))[0]
    idx = np.arange(n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = _mix(key + (idx * np.uint64(2) + np.uint64(lane)) * np.uint64(0x9E3779B97F4A7C15))
    return ((z >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: str, shape, sigma: float = 1.0, mean: float = 0.0) -> np.ndarray:
    """N(mean, sigma^2) float64 array by Box-Muller on two counter-based uniforms."""
    n = int(np.prod(shape)) if len(shape) else 1
    u1 = _u01(seed, stream, 0, n)
    u2 = _u01(seed, stream, 1, n)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (mean + sigma * z).reshape(shape)


def uniform_int(seed: int, stream: str, shape, hi: int) -> np.ndarray:
    n = int(np.prod(shape)) if len(shape) else 1
    u = _u01(seed, stream, 0, n)
    return np.minimum((u * hi).astype(np.int32), hi - 1).reshape(shape)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit pattern (uint16)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Values of `a` rounded to bfloat16, returned as float64."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a)).astype(np.float64).reshape(np.shape(a))


def _store(a: np.ndarray, dtype: str, low_precision: bool) -> np.ndarray:
    """Round to what the device will hold: bf16 for low-precision tensors in bf16 mode, else fp32."""
    if dtype == "bf16" and low_precision:
        return round_bf16(a)
    return a.astype(np.float32).astype(np.float64)


def _gen_tensor(seed, prefix, spec, dtype):
    s = f"{prefix}/{spec.name}"
    if spec.kind == "conv":
        return _store(normal(seed, s, spec.shape, np.sqrt(2.0 / spec.fan_in)), dtype, True)
    if spec.kind == "fc_w":
        return _store(normal(seed, s, spec.shape, np.sqrt(2.0 / spec.fan_in)), dtype, False)
    if spec.kind == "bn_gamma":
        return _store(normal(seed, s, spec.shape, 0.1, 1.0), dtype, False)
    return _store(normal(seed, s, spec.shape, 0.1), dtype, False)   # bn_beta, fc_b


def make_params(net: NetDesc, k: int):
    """Parameter tensors of module k (float64 values exactly representable in the storage type).

    Conv filters: Kaiming-normal N(0, 2/fan_in), stored in the net's dtype.  BN gamma = 1 + N(0,0.1^2),
    BN beta = N(0,0.1^2), FC weight Kaiming-normal, FC bias N(0,0.1^2): all kept in fp32.
    """
    return [_gen_tensor(net.seed, f"module{k}", sp, net.dtype) for sp in module_tensor_specs(net.modules[k])]


def make_aux_params(net: NetDesc, j: int):
    """Parameters of the AuxNet block that generates x_{j+1}."""
    return [_gen_tensor(net.seed, f"aux{j}", sp, net.dtype) for sp in aux_tensor_specs(net.aux[j])]


def make_image(net: NetDesc) -> np.ndarray:
    m = net.modules[0]
    return _store(normal(net.seed, "image", (m.N, m.H, m.W, m.C)), net.dtype, True)


def make_labels(net: NetDesc) -> np.ndarray:
    m = net.modules[-1]
    return uniform_int(net.seed, "labels", (m.N,), m.n_classes)


def make_noise(net: NetDesc, name: str, shape, sigma: float) -> np.ndarray:
    """Unrounded N(0, sigma^2) perturbation (callers round the perturbed tensor to the storage type)."""
    return normal(net.seed, name, shape, sigma)
