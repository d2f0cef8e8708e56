"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no posit arithmetic: everything here is IEEE floats (to be rounded to a
posit format by whichever side consumes them) and layer shapes.  The shapes are
those of the paper's workloads (28x28x1 images through a LeNet-5-like network,
32x32x3 images through a CifarNet-like network, Sec. 4); the values are synthetic
stand-ins drawn from numpy's PCG64 generator, not items of any dataset.
"""
import numpy as np

BASE_SEED = 2105000530  # config c uses BASE_SEED + c


def rng_for(config, stream=0):
    return np.random.default_rng([BASE_SEED + int(config), int(stream)])


def normal_matrix(config, stream, shape, sigma=1.0):
    """float32 N(0, sigma^2) draws."""
    return (rng_for(config, stream).standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def uniform_tensor(config, stream, shape):
    """float32 U(0, 1) draws."""
    return rng_for(config, stream).random(size=shape, dtype=np.float32)


def with_regime_extremes(x, config, stream, fraction=0.01, log2_range=28.0):
    """Replace exactly floor(fraction * size) entries (chosen without replacement)
    by +-2^U, U uniform in [-log2_range, log2_range]: exercises the long-regime ends
    of posit<16,1>.  Returns float64 so that 2^+-28 scale values stay exact enough
    to be rounded by the consumer."""
    r = rng_for(config, stream)
    flat = np.array(x, dtype=np.float64).reshape(-1)
    n = int(fraction * flat.size)
    idx = r.choice(flat.size, size=n, replace=False)
    mag = np.exp2(r.uniform(-log2_range, log2_range, size=n))
    sign = np.where(r.random(size=n) < 0.5, -1.0, 1.0)
    flat[idx] = sign * mag
    return flat.reshape(np.shape(x))


def gemm_operands(config, S, sigma=1.0, extremes=False):
    """A[S,S], B[S,S] for the square GEMM configurations."""
    if isinstance(S, int):
        S = (S, S, S)
    M, N, K = S
    A = normal_matrix(config, 0, (M, K), sigma)
    B = normal_matrix(config, 1, (K, N), sigma)
    if extremes:
        A = with_regime_extremes(A, config, 2)
        B = with_regime_extremes(B, config, 3)
    return A, B


def he_normal(config, stream, shape):
    """He-normal weights: sigma = sqrt(2 / fan_in); shape is (out, in[, kh, kw])."""
    fan_in = int(np.prod(shape[1:]))
    return normal_matrix(config, stream, shape, np.sqrt(2.0 / fan_in))


# Layer lists.  conv: (Cin, Cout, kernel, pad); pool: window 2; fc: (in, out).
LENET = dict(
    config=3, batch=64, input=(1, 28, 28), input_dist="uniform",
    layers=[("conv", 1, 6, 5, 2), ("relu",), ("avgpool",), ("conv", 6, 16, 5, 0), ("relu",), ("avgpool",),
            ("flatten",), ("fc", 400, 120), ("relu",), ("fc", 120, 84), ("relu",), ("fc", 84, 10)],
)
CIFARNET = dict(
    config=4, batch=128, input=(3, 32, 32), input_dist="normal",
    layers=[("conv", 3, 32, 3, 1), ("relu",), ("conv", 32, 32, 3, 1), ("relu",), ("maxpool",),
            ("conv", 32, 64, 3, 1), ("relu",), ("conv", 64, 64, 3, 1), ("relu",), ("maxpool",),
            ("conv", 64, 128, 3, 1), ("relu",), ("maxpool",), ("flatten",), ("fc", 2048, 10)],
)


def network_inputs(net, batch=None):
    """Input batch, per-layer float32 weights/biases (He-normal, zero bias) and labels."""
    cfg = net["config"]
    n = batch or net["batch"]
    shape = (n,) + tuple(net["input"])
    x = uniform_tensor(cfg, 0, shape) if net["input_dist"] == "uniform" else normal_matrix(cfg, 0, shape)
    params = []
    stream = 10
    for layer in net["layers"]:
        if layer[0] == "conv":
            _, cin, cout, k, _pad = layer
            params.append((he_normal(cfg, stream, (cout, cin, k, k)), np.zeros(cout, dtype=np.float32)))
            stream += 1
        elif layer[0] == "fc":
            _, fin, fout = layer
            params.append((he_normal(cfg, stream, (fout, fin)), np.zeros(fout, dtype=np.float32)))
            stream += 1
    labels = rng_for(cfg, 1).integers(0, 10, size=n)
    return x, params, labels
