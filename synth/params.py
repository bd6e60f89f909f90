"""Seeded random parameters.  Values only; the caller hands them to whichever implementation it tests."""
import numpy as np

from .shapes import ModelShape, param_specs


def init_params(shape: ModelShape, seed: int, *, generic: bool = False):
    """Return {name: float64 array}.

    Default recipe: embedding ~ N(0, 1/sqrt(d)), matrices ~ U(+-sqrt(6/(in+out))), biases 0,
    LayerNorm gain 1 and shift 0.  With generic=True biases, gains and shifts are random as well, so that a
    test exercises every term (a zero bias would hide a dropped bias gradient).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    d = shape.d_model
    out = {}
    for name, shp in param_specs(shape):
        if name == "embed" or (name.startswith("embed.") and not name.endswith(".proj")):
            a = rng.normal(0.0, shp[1] ** -0.5, size=shp)
        elif len(shp) == 2:
            lim = (6.0 / (shp[0] + shp[1])) ** 0.5
            a = rng.uniform(-lim, lim, size=shp)
        elif name.endswith(".g"):
            a = 1.0 + (rng.uniform(-0.3, 0.3, size=shp) if generic else 0.0) * np.ones(shp)
        else:
            a = rng.uniform(-0.2, 0.2, size=shp) if generic else np.zeros(shp)
        out[name] = np.ascontiguousarray(a, dtype=np.float64)
    return out
