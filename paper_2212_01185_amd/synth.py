"""Seeded synthetic inputs: test images and weight blobs.

This module holds no arithmetic of the coding method itself.  It only draws
random numbers and serialises them, so that the CPU oracle and the HIP library
can be fed byte-identical inputs without sharing any code of the method.

Images stand in for the photographic test crops the paper times on (Sec. IV-A,
Table II): smooth coloured structure plus a little sensor-like noise.
Weights stand in for the trained network of Sec. III-B (no trained weights
exist here): He-initialised, seeded, pre-rounded to bf16 so that an fp64 CPU
evaluation and a bf16 matrix-core evaluation see the same numbers.
"""
from __future__ import annotations

import struct
from dataclasses import dataclass

import numpy as np

# --------------------------------------------------------------------------
# workload table (the five measured configurations)
# --------------------------------------------------------------------------


@dataclass(frozen=True)
class ImageSpec:
    width: int
    height: int
    n_blobs: int
    sigma_lo: float
    sigma_hi: float
    value_noise: bool = False


@dataclass(frozen=True)
class Workload:
    name: str
    n_images: int
    spec: ImageSpec


WORKLOADS = {
    0: Workload("64x64", 1, ImageSpec(64, 64, 8, 4.0, 16.0)),
    1: Workload("768x512", 1, ImageSpec(768, 512, 32, 8.0, 64.0)),
    2: Workload("24x768x512", 24, ImageSpec(768, 512, 32, 8.0, 64.0)),
    3: Workload("2048x1365", 1, ImageSpec(2048, 1365, 128, 16.0, 256.0, value_noise=True)),
    4: Workload("4096x2160", 1, ImageSpec(4096, 2160, 512, 32.0, 512.0)),
}


def _value_noise(rng: np.random.Generator, height: int, width: int, cell: int) -> np.ndarray:
    """Bilinear interpolation of a coarse random lattice (one octave), in [-1, 1]."""
    gh = height // cell + 2
    gw = width // cell + 2
    lattice = rng.uniform(-1.0, 1.0, size=(gh, gw, 3))
    ys = np.arange(height) / cell
    xs = np.arange(width) / cell
    y0 = ys.astype(np.int64)
    x0 = xs.astype(np.int64)
    fy = (ys - y0)[:, None, None]
    fx = (xs - x0)[None, :, None]
    a = lattice[y0][:, x0]
    b = lattice[y0][:, x0 + 1]
    c = lattice[y0 + 1][:, x0]
    d = lattice[y0 + 1][:, x0 + 1]
    return (a * (1 - fx) + b * fx) * (1 - fy) + (c * (1 - fx) + d * fx) * fy


def make_image(seed: int, spec: ImageSpec) -> np.ndarray:
    """One uint8 image of shape [height, width, 3] (rows, columns, RGB).

    Sum of Gaussian blobs + one linear gradient + N(0, 3) noise per sub-pixel
    (+ two octaves of value noise when the spec asks), rounded and clipped.
    Blob amplitudes are drawn from U(0, 255) per channel and then scaled by
    min(1, 1.5 / coverage), coverage = n_blobs * 2*pi*E[sigma^2] / (W*H), so
    that specs with many wide blobs do not saturate to a flat white image.
    """
    rng = np.random.default_rng(seed)
    h, w = spec.height, spec.width
    cx = rng.uniform(0, w, spec.n_blobs)
    cy = rng.uniform(0, h, spec.n_blobs)
    sg = rng.uniform(spec.sigma_lo, spec.sigma_hi, spec.n_blobs)
    amp = rng.uniform(0, 255, (spec.n_blobs, 3))
    mean_sq = (spec.sigma_lo ** 2 + spec.sigma_lo * spec.sigma_hi + spec.sigma_hi ** 2) / 3.0
    coverage = spec.n_blobs * 2 * np.pi * mean_sq / (w * h)
    amp *= min(1.0, 1.5 / coverage)

    # separable blobs: exp(-(dx^2+dy^2)/2s^2) = gy * gx, summed as one matrix product per channel
    gy = np.exp(-0.5 * ((np.arange(h)[:, None] - cy[None, :]) / sg[None, :]) ** 2)   # [h, nb]
    gx = np.exp(-0.5 * ((np.arange(w)[None, :] - cx[:, None]) / sg[:, None]) ** 2)   # [nb, w]
    img = np.empty((h, w, 3), dtype=np.float64)
    for ch in range(3):
        img[:, :, ch] = gy @ (gx * amp[:, ch:ch + 1])

    # linear gradient: random direction, peak-to-peak U(0, 128) per channel
    theta = rng.uniform(0, 2 * np.pi)
    p2p = rng.uniform(0, 128, 3)
    ramp = (np.cos(theta) * (np.arange(w)[None, :] / max(w - 1, 1))
            + np.sin(theta) * (np.arange(h)[:, None] / max(h - 1, 1)))
    ramp = (ramp - ramp.min()) / max(ramp.max() - ramp.min(), 1e-12)
    img += ramp[:, :, None] * p2p[None, None, :]

    if spec.value_noise:
        img += 20.0 * _value_noise(rng, h, w, 64)
        img += 10.0 * _value_noise(rng, h, w, 32)

    img += rng.normal(0.0, 3.0, size=(h, w, 3))
    return np.clip(np.rint(img), 0, 255).astype(np.uint8)


def make_batch(config: int, n_images: int | None = None) -> np.ndarray:
    """uint8 [n, H, W, 3] for one of the five workloads (image i uses seed i)."""
    wl = WORKLOADS[config]
    n = wl.n_images if n_images is None else n_images
    return np.stack([make_image(s, wl.spec) for s in range(n)], axis=0)


# --------------------------------------------------------------------------
# weight blob
# --------------------------------------------------------------------------

BLOB_MAGIC = 0x57434350        # "PCCW" little-endian
BLOB_VERSION = 1
BLOB_HEADER_BYTES = 64         # 16 little-endian uint32 words
ACT_RELU, ACT_LEAKY = 0, 1
DIST_GAUSSIAN, DIST_LOGISTIC = 0, 1

DEFAULT_DIMS = (30, 160, 160, 128, 60)
DEFAULT_K = 5
DEFAULT_NBHD = 10
DEFAULT_DELAY = 2

# the paper's own network (Sec. III-B and the hyper-parameter table of Sec. IV-E): first layer on the
# 12 unmasked taps of a 5x5 window, four more layers of 128 filters, LeakyReLU, K = 3 mixtures
PAPER_DIMS = (36, 128, 128, 128, 128, 36)
PAPER_K = 3
PAPER_NBHD = 12
PAPER_DELAY = 3


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32)


def make_weights(seed: int = 0, dims=DEFAULT_DIMS, sharp: bool = False):
    """He-initialised layers: W ~ N(0, 2/fan_in) rounded to bf16, biases zero.

    ``sharp=True`` is a test-only variant whose head is damped (last-layer
    weights x0.1) and biased (means 0.5, log-sigmas -4) so that the mixtures
    are narrow and many symbols land in the tails (frequency 1).
    Returns a list of (W[out, in] float32, b[out] float32).
    """
    rng = np.random.default_rng(seed)
    layers = []
    for fan_in, fan_out in zip(dims[:-1], dims[1:]):
        w = rng.normal(0.0, np.sqrt(2.0 / fan_in), size=(fan_out, fan_in)).astype(np.float32)
        b = np.zeros(fan_out, dtype=np.float32)
        layers.append([w, b])
    if sharp:
        k = dims[-1] // 12
        w, b = layers[-1]
        w *= 0.1
        for ch in range(3):
            b[3 * k * ch + k: 3 * k * ch + 2 * k] = 0.5
            b[3 * k * ch + 2 * k: 3 * k * ch + 3 * k] = -4.0
    return [(round_to_bf16(w), b) for w, b in layers]


def pack_blob(layers, k=DEFAULT_K, nbhd=DEFAULT_NBHD, delay=DEFAULT_DELAY,
              act=ACT_RELU, dist=DIST_GAUSSIAN) -> bytes:
    """Serialise: 64-byte header, then per layer W (row-major [out][in] fp32) and b (fp32).

    Header words: magic, version, n_layers, dims[0..7] (unused = 0), K,
    neighbourhood size, wavefront delay per row, activation id, distribution id.
    """
    dims = [layers[0][0].shape[1]] + [w.shape[0] for w, _ in layers]
    if len(dims) > 8:
        raise ValueError("at most 7 layers")
    words = [BLOB_MAGIC, BLOB_VERSION, len(layers)] + dims + [0] * (8 - len(dims)) \
        + [k, nbhd, delay, act, dist]
    out = [struct.pack("<16I", *words)]
    for w, b in layers:
        out.append(np.ascontiguousarray(w, dtype="<f4").tobytes())
        out.append(np.ascontiguousarray(b, dtype="<f4").tobytes())
    return b"".join(out)


def make_blob(seed: int = 0, sharp: bool = False, dist: int = DIST_GAUSSIAN) -> bytes:
    """The weight blob every workload uses (seed 0, default shape)."""
    return pack_blob(make_weights(seed, DEFAULT_DIMS, sharp=sharp), dist=dist)


def make_paper_blob(seed: int = 0, sharp: bool = False, dist: int = DIST_GAUSSIAN) -> bytes:
    """A weight blob of the paper's network shape (He-initialised: no trained weights exist here)."""
    return pack_blob(make_weights(seed, PAPER_DIMS, sharp=sharp), k=PAPER_K, nbhd=PAPER_NBHD, delay=PAPER_DELAY,
                     act=ACT_LEAKY, dist=dist)


def make_predictor_weights(sigma_levels: float = 6.0):
    """Hand-structured weights of the default shape: every mixture component of channel ch is a Gaussian
    around the plane prediction left + up - upleft of that channel, with a fixed width of
    ``sigma_levels`` grey levels; no coupling.  All weights are 0, 1 or -1 (bf16-exact).  Not trained:
    a stand-in that makes the coder actually compress smooth images, and whose head outputs have a
    closed form (a pin for gather order, layer chaining and head layout)."""
    dims = DEFAULT_DIMS
    k = DEFAULT_K
    layers = [[np.zeros((o, i), dtype=np.float32), np.zeros(o, dtype=np.float32)] for i, o in zip(dims[:-1], dims[1:])]
    left, up, upleft = 9, 6, 5                       # neighbour indices in raster order: (0,-1), (-1,0), (-1,-1)
    for ch in range(3):
        for sign, unit in ((1.0, 2 * ch), (-1.0, 2 * ch + 1)):    # positive and negative part survive the ReLUs
            layers[0][0][unit, 3 * left + ch] = sign
            layers[0][0][unit, 3 * up + ch] = sign
            layers[0][0][unit, 3 * upleft + ch] = -sign
            layers[1][0][unit, unit] = 1.0
            layers[2][0][unit, unit] = 1.0
        for comp in range(k):
            layers[3][0][3 * k * ch + k + comp, 2 * ch] = 1.0        # mean = positive part - negative part
            layers[3][0][3 * k * ch + k + comp, 2 * ch + 1] = -1.0
            layers[3][1][3 * k * ch + 2 * k + comp] = np.log(sigma_levels / 256.0)
    return [(w, b) for w, b in layers]


def make_predictor_blob(sigma_levels: float = 6.0) -> bytes:
    return pack_blob(make_predictor_weights(sigma_levels))


DELTA_R_LEVEL, DELTA_G_LEVELS, DELTA_B_LEVEL = 100, (50, 200), 255


def make_delta_blob() -> bytes:
    """Test-only weights of the default shape that drive the coder to its extreme frequencies: all weights 0, so
    every pixel gets the same three distributions from the head biases alone; every log-sigma is -8 (the lower
    clamp: sigma = 0.086 grey levels, all of a component's mass in one bin).  R: every component sits on the
    centre of bin 100, so level 100 takes the whole scaled mass (frequency 65,281 with the one-count floor of
    every bin) and every other level has frequency 1.  G: three components on bin 50, two on bin 200, equal
    weights (frequencies about 0.6 and 0.4 of the total).  B: means far above the range (3.0 = 768 grey levels),
    so level 255 takes the open upper tail (65,281) and all others frequency 1.  No coupling."""
    dims, k = DEFAULT_DIMS, DEFAULT_K
    layers = [[np.zeros((o, i), dtype=np.float32), np.zeros(o, dtype=np.float32)] for i, o in zip(dims[:-1], dims[1:])]
    b = layers[-1][1]
    for ch in range(3):
        b[3 * k * ch + 2 * k: 3 * k * ch + 3 * k] = -8.0
    b[k:2 * k] = DELTA_R_LEVEL / 256.0
    b[3 * k + k: 3 * k + k + 3] = DELTA_G_LEVELS[0] / 256.0
    b[3 * k + k + 3: 3 * k + 2 * k] = DELTA_G_LEVELS[1] / 256.0
    b[6 * k + k: 6 * k + 2 * k] = 3.0
    return pack_blob([(w, bb) for w, bb in layers])


def make_delta_image(seed: int, n: int, h: int, w: int) -> np.ndarray:
    """uint8 [n, h, w, 3] for the delta weights: runs of the levels the distributions sit on (frequencies near
    the maximum: the coder state hardly moves), runs of uniformly random pixels (frequency 1: a renormalisation
    word every other symbol), and single pixels of either kind, in seeded order."""
    rng = np.random.default_rng(seed)
    flat = np.empty((n * h * w, 3), dtype=np.uint8)
    at = 0
    heavy = bool(rng.integers(2))
    while at < len(flat):
        run = int(rng.choice([1, 2, 7, 40, 333]))
        run = min(run, len(flat) - at, max(1, len(flat) // 5))      # both kinds occur in any image of a few pixels
        heavy = not heavy
        if heavy:
            flat[at:at + run, 0] = DELTA_R_LEVEL
            flat[at:at + run, 1] = rng.choice(DELTA_G_LEVELS, run)
            flat[at:at + run, 2] = DELTA_B_LEVEL
        else:
            flat[at:at + run] = rng.integers(0, 256, (run, 3), dtype=np.uint8)
        at += run
    return flat.reshape(n, h, w, 3)


PROBE_TAPS = (11, 4, 5)     # of the 12 neighbours in raster order: (0,-1), (-2,+2), (-1,-2)


def make_tap_probe_blob(delay: int = PAPER_DELAY) -> bytes:
    """The paper's network shape with hand-set weights: the mean of component k of channel ch is the
    value of neighbour PROBE_TAPS[k], channel ch, passed unchanged through the four LeakyReLU layers
    (inputs are non-negative); logits and coupling 0, sigma 6 grey levels.  Closed-form head outputs
    that pin the order of the 12 neighbours (delay 3) and the copies of the diagonal order (delay 1)."""
    dims = PAPER_DIMS
    layers = [[np.zeros((o, i), dtype=np.float32), np.zeros(o, dtype=np.float32)] for i, o in zip(dims[:-1], dims[1:])]
    for k, tap in enumerate(PROBE_TAPS):
        for ch in range(3):
            unit = 3 * k + ch
            layers[0][0][unit, 3 * tap + ch] = 1.0
            for l in (1, 2, 3):
                layers[l][0][unit, unit] = 1.0
            layers[4][0][3 * PAPER_K * ch + PAPER_K + k, unit] = 1.0
            layers[4][1][3 * PAPER_K * ch + 2 * PAPER_K + k] = np.log(6.0 / 256.0)
    return pack_blob([(w, b) for w, b in layers], k=PAPER_K, nbhd=PAPER_NBHD, delay=delay, act=ACT_LEAKY)


def make_diagonal_blob(seed: int = 0, sharp: bool = False, dist: int = DIST_GAUSSIAN) -> bytes:
    """The paper's network shape for the diagonal decoding order (Sec. III-C, Eq. (7)): same layers and
    12-pixel input, rows trail by one column (delay 1), three inputs are copies (the coder's business)."""
    return pack_blob(make_weights(seed, PAPER_DIMS, sharp=sharp), k=PAPER_K, nbhd=PAPER_NBHD, delay=1,
                     act=ACT_LEAKY, dist=dist)


# The shapes of the paper's ablation study (Sec. IV-E: one hyper-parameter of (K, C, L) = (3, 128, 5) changed at a
# time), all of which the GPU library takes: name -> (mixtures K, filters C, layers L).
ABLATION_SHAPES = {"fewer_layers": (3, 128, 4), "fewer_filters": (3, 64, 5), "more_mixtures": (5, 128, 5),
                   "most_mixtures": (7, 128, 5), "more_layers": (3, 128, 6),
                   "more_filters": (3, 192, 5)}


def ablation_dims(k: int, c: int, n_layers: int):
    """Layer widths of the paper's network with K mixtures, C filters and L layers: 36, C x (L-1), 12 K."""
    return (PAPER_DIMS[0],) + (c,) * (n_layers - 1) + (12 * k,)


def make_ablation_blob(k: int, c: int, n_layers: int, seed: int = 0, sharp: bool = False,
                       dist: int = DIST_GAUSSIAN) -> bytes:
    """A weight blob of one of the ablation shapes (He-initialised), wavefront order."""
    return pack_blob(make_weights(seed, ablation_dims(k, c, n_layers), sharp=sharp), k=k, nbhd=PAPER_NBHD,
                     delay=PAPER_DELAY, act=ACT_LEAKY, dist=dist)


def param_count(dims) -> int:
    """Weights + biases of a fully connected stack with these layer widths."""
    return sum(i * o + o for i, o in zip(dims[:-1], dims[1:]))
