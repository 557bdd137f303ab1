"""Seeded initial parameter values (values only; no model arithmetic)."""
import numpy as np

# name -> shape as a function of (N, R, d, h)
MLP_PARAM_NAMES = ("W1", "b1", "W2", "b2",      # projection
                   "V1", "c1", "V2", "c2",      # negation
                   "U1", "u1", "U2", "u2")      # intersection attention
PARAM_NAMES = ("E", "R") + MLP_PARAM_NAMES


def param_shapes(N, R, d, h, d_sem=0):
    s = {"E": (N, d), "R": (R, d)}
    for a, b, c, e in (("W1", "b1", "W2", "b2"), ("V1", "c1", "V2", "c2"),
                       ("U1", "u1", "U2", "u2")):
        s[a] = (h, d)
        s[b] = (h,)
        s[c] = (d, h)
        s[e] = (d,)
    if d_sem:
        s["Wp"] = (d, d_sem)
    return s


def make_params(N, R, d, h, seed, d_sem=0, scale=0.1):
    """Every tensor (biases too) U(-scale, scale), fp32, in a fixed draw order."""
    rng = np.random.default_rng(seed)
    out = {}
    for name, shape in param_shapes(N, R, d, h, d_sem).items():
        out[name] = ((rng.random(shape, np.float32) * 2 - 1) * scale).astype(np.float32)
    return out


BOX_PARAM_NAMES = ("E", "R", "Ro", "V1", "c1", "V2", "c2", "U1", "u1", "U2", "u2")


def make_box_params(N, R, d, h, seed, scale=0.1):
    """Tensors of the box family: E and R (centres), Ro (relation offsets), the offset MLP
    V1 c1 V2 c2 and the centre-attention MLP U1 u1 U2 u2.  Everything U(-scale, scale) except
    Ro, which is U(-scale/4, scale) so that most, not all, of its entries are positive."""
    rng = np.random.default_rng(seed)
    shapes = {"E": (N, d), "R": (R, d), "Ro": (R, d)}
    for a, b, c, e in (("V1", "c1", "V2", "c2"), ("U1", "u1", "U2", "u2")):
        shapes.update({a: (h, d), b: (h,), c: (d, h), e: (d,)})
    out = {}
    for name in BOX_PARAM_NAMES:
        u = rng.random(shapes[name], np.float32)
        lo = -scale / 4 if name == "Ro" else -scale
        out[name] = (lo + u * (scale - lo)).astype(np.float32)
    return out


def make_sem_features(N, d_sem, seed, chunk=1 << 16):
    """[N, d_sem] frozen features: N(0,1) rows, L2-normalised, rounded to bf16.

    Returned as uint16 holding the bf16 bit patterns (round-to-nearest-even).
    """
    rng = np.random.default_rng(seed)
    out = np.empty((N, d_sem), np.uint16)
    for lo in range(0, N, chunk):
        hi = min(N, lo + chunk)
        x = rng.standard_normal((hi - lo, d_sem), np.float32)
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        bits = x.view(np.uint32)
        bits = bits + 0x7FFF + ((bits >> 16) & 1)
        out[lo:hi] = (bits >> 16).astype(np.uint16)
    return out
