"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only counter-based random draws (numpy's
Philox) with the shapes and value distributions of the paper's workload
(Sec. 3.2: 224x224 images, 1000 classes, per-worker mini-batch 16 or 32),
standing in for ImageNet, which is not available.  All float tensors that the
mixed-precision path stores in FP16 are drawn in float32 and then rounded to
binary16-representable values, so that both sides start from identical numbers.
"""
import numpy as np

BASE_SEED = 0x181105233


def rng(stream):
    return np.random.Generator(np.random.Philox(key=BASE_SEED + int(stream)))


def normal_f16(stream, shape, std=1.0):
    """N(0, std^2) values representable in binary16, returned as float32."""
    a = rng(stream).standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return a.astype(np.float16).astype(np.float32)


def normal_f32(stream, shape, std=1.0):
    return rng(stream).standard_normal(size=shape, dtype=np.float32) * np.float32(std)


def labels(stream, batch, classes=1000):
    return rng(stream).integers(0, classes, size=batch, dtype=np.int32)


def he_normal_f16(stream, shape, fan_in):
    return normal_f16(stream, shape, np.sqrt(2.0 / fan_in))


def flat_params(stream, segments):
    """Flat float32 master-parameter vector for a list of (kind, offset, count, fan_in).

    kind 0 (conv filter) and 3 (FC weight): He-normal, std = sqrt(2/fan_in);
    kind 1 (BN gamma): 1; kind 2 (BN beta) and 4 (FC bias): 0.
    """
    total = max(off + cnt for _, off, cnt, _ in segments)
    w = np.zeros(total, np.float32)
    for i, (kind, off, cnt, fan_in) in enumerate(segments):
        if kind in (0, 3):
            w[off:off + cnt] = he_normal_f16(stream * 1000 + i, (cnt,), fan_in)
        elif kind == 1:
            w[off:off + cnt] = 1.0
    return w
