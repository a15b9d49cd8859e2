"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds none of the method's arithmetic: it only draws random numbers of the requested shapes.
Weights: every conv / linear weight and bias ~ N(0, 0.02); normalisation gains 1, offsets 0.
Latent and text embedding ~ N(0, 1).  Generator: NumPy PCG64 seeded per tensor family.
"""
import numpy as np

SEED_WEIGHTS, SEED_LATENT, SEED_TEXT, SEED_POOLED = 1000, 2000, 3000, 4000


def _is_norm_gain(name):
    return name.endswith(".g")


def _is_norm_offset(name):
    last = name.rsplit(".", 2)
    return name.endswith(".b") and len(last) >= 2 and (last[-2].startswith("gn") or last[-2].startswith("ln"))


def make_weights(manifest, seed=SEED_WEIGHTS, std=0.02, bf16_exact=False):
    """manifest: iterable of (name, shape).  Returns {name: float32 array}.

    bf16_exact rounds every drawn value to the nearest bfloat16 (ties to even) so that a bf16
    and an fp64 consumer start from identical numbers.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name, shape in manifest:
        if _is_norm_gain(name):
            a = np.ones(shape, np.float32)
        elif _is_norm_offset(name):
            a = np.zeros(shape, np.float32)
        else:
            a = (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)
            if bf16_exact:
                a = round_to_bf16(a)
        out[name] = a
    return out


def round_to_bf16(a):
    """Nearest-even rounding of float32 values to bfloat16 precision, returned as float32."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32).reshape(np.shape(a))


def make_latent(channels, h, w, seed=SEED_LATENT):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((channels, h, w), dtype=np.float32)


def make_video_latent(frames, channels, h, w, seed=SEED_LATENT):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((frames, channels, h, w), dtype=np.float32)


def make_text(batch, ctx_len, ctx_dim, seed=SEED_TEXT):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((batch, ctx_len, ctx_dim), dtype=np.float32)


def make_pooled(batch, dim, seed=SEED_POOLED):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((batch, dim), dtype=np.float32)


def make_array(shape, seed, scale=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)).astype(np.float32)
