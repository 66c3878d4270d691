"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no layer arithmetic: only a counter-based random generator, the value
distributions of the workloads, and bf16 rounding of generated values.  The
same bytes are handed to the GPU library and to the CPU oracle.

Generator: element i of tensor `name` is SplitMix64's i-th output for the state
seed ^ fnv1a64(name); uniforms use the top 53 bits; normals use Box-Muller on
the uniform pair (2i, 2i+1).
"""
import numpy as np

SEED = 20211210
_G = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 20


def fnv1a64(name: str) -> int:
    h = 0xCBF29CE484222325
    for b in name.encode():
        h = ((h ^ b) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _u01(base: int, idx):
    """Uniform in (0,1) for counters idx (uint64 array)."""
    with np.errstate(over="ignore"):
        z = np.uint64(base) + (idx + np.uint64(1)) * _G
        u = _mix(z) >> np.uint64(11)
    return (u.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _base(name, seed):
    return (int(seed) ^ fnv1a64(name)) & 0xFFFFFFFFFFFFFFFF


def _fill_chunks(n, fill):
    """Run fill(start, end) over [0, n) in chunks; large tensors use a few threads (every element depends
    on its own counter only, so the values do not depend on how the range is cut up)."""
    spans = [(s, min(n, s + _CHUNK)) for s in range(0, n, _CHUNK)]
    if len(spans) < 4:
        for s, e in spans:
            fill(s, e)
        return
    import os
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1))) as ex:
        list(ex.map(lambda se: fill(*se), spans))


def uniform(name, shape, lo=-1.0, hi=1.0, seed=SEED):
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    b = _base(name, seed)

    def fill(s, e):
        idx = np.arange(s, e, dtype=np.uint64)
        out[s:e] = lo + (hi - lo) * _u01(b, idx)
    _fill_chunks(n, fill)
    return out.reshape(shape)


def normal(name, shape, std=1.0, seed=SEED):
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    b = _base(name, seed)

    def fill(s, e):
        idx = np.arange(s, e, dtype=np.uint64)
        u1 = _u01(b, idx * np.uint64(2))
        u2 = _u01(b, idx * np.uint64(2) + np.uint64(1))
        out[s:e] = std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    _fill_chunks(n, fill)
    return out.reshape(shape)


# ---- bf16 storage helpers (round-to-nearest-even), values kept as uint16 bits ----
def f32_to_bf16_bits(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(a):
    """fp32 array holding the bf16-rounded values of `a`."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# ---- tensors of one layer, by the recipes of the workload configurations ----
def conv_tensors(tag, n, h, w, c, k, r, s, dist="he_normal", bias=True, seed=SEED):
    """x, w, b (fp32 values) for one conv layer.

    dist = "he_normal": x ~ N(0,1), w ~ N(0, 2/(r*s*c));
    dist = "he_uniform": x ~ U[-1,1], w ~ U[-1,1]*sqrt(6/(r*s*c)).
    Bias ~ U[-0.1,0.1].  The sample index is part of the counter, so the first
    n' < n samples of a larger batch are the batch-n' tensors.
    """
    fan_in = r * s * c
    if dist == "he_normal":
        x = normal(f"{tag}/x", (n, h, w, c), 1.0, seed)
        wt = normal(f"{tag}/w", (k, r, s, c), float(np.sqrt(2.0 / fan_in)), seed)
    elif dist == "he_uniform":
        x = uniform(f"{tag}/x", (n, h, w, c), -1.0, 1.0, seed)
        a = float(np.sqrt(6.0 / fan_in))
        wt = uniform(f"{tag}/w", (k, r, s, c), -a, a, seed)
    else:
        raise ValueError(dist)
    b = uniform(f"{tag}/b", (k,), -0.1, 0.1, seed) if bias else None
    return x, wt, b


def upstream_grad(tag, shape, seed=SEED):
    return normal(f"{tag}/dy", shape, 1.0, seed)


def linear_tensors(tag, n, in_f, out_f, bias=True, seed=SEED):
    x = normal(f"{tag}/x", (n, in_f), 1.0, seed)
    W = normal(f"{tag}/w", (out_f, in_f), float(np.sqrt(2.0 / in_f)), seed)
    b = uniform(f"{tag}/b", (out_f,), -0.1, 0.1, seed) if bias else None
    return x, W, b
