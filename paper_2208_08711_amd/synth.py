"""Seeded synthetic image generators for the benchmark configurations.

This module holds no codec arithmetic: it only makes uint8 RGB images (and crop
parameters) whose shapes and rough statistics stand in for the paper's
workloads (Section 5.1, Table "batch": Cityscapes-sized street scenes in
batches of 32-48; smaller photo-like images).  The real datasets are not used.
Both the CPU oracle's tests and the GPU path's tests and benchmark draw their
inputs from here, so that they see identical bytes.

Randomness is a counter-based generator written out below (a 64-bit mixing
function of seed and counter), so results do not depend on a library's
distribution code.  Uniforms use the top 53 bits; Gaussians use Box-Muller.
Image k of configuration c uses seed 1000*c + k (configuration 1: seed 0).
"""
import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


class Stream:
    """Counter-based stream: value i of stream (seed, lane) is a pure function of them."""

    def __init__(self, seed, lane=0):
        with np.errstate(over="ignore"):
            self.key = _mix(np.array([np.uint64(seed) * _GOLD + np.uint64(lane) + np.uint64(1)],
                                     dtype=np.uint64))[0]
        self.counter = 0

    def bits(self, n):
        idx = np.arange(self.counter, self.counter + n, dtype=np.uint64)
        self.counter += n
        with np.errstate(over="ignore"):
            return _mix((idx + np.uint64(1)) * _GOLD + self.key)

    def uniform(self, n):
        return (self.bits(n) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))

    def integers(self, lo, hi, n=1):
        """n integers uniform in lo..hi inclusive."""
        u = self.uniform(n)
        return (lo + np.floor(u * (hi - lo + 1))).astype(np.int64)

    def normal(self, n):
        m = (n + 1) // 2
        u1 = 1.0 - self.uniform(m)          # (0, 1]
        u2 = self.uniform(m)
        r = np.sqrt(-2.0 * np.log(u1))
        out = np.empty(2 * m, dtype=np.float64)
        out[0::2] = r * np.cos(2.0 * np.pi * u2)
        out[1::2] = r * np.sin(2.0 * np.pi * u2)
        return out[:n]

    def bytes(self, n):
        m = (n + 7) // 8
        return self.bits(m).view(np.uint8)[:n].copy()


def _to_u8(x):
    return np.clip(np.rint(x), 0, 255).astype(np.uint8)


def gradient_noise(seed, width, height, sigma, span=None):
    """Horizontal + vertical linear gradient plus Gaussian noise.

    span=None: slopes 1.5 per pixel from 32 (+20 per channel); otherwise each channel
    is a differently oriented diagonal ramp spanning 0..span over the image."""
    s = Stream(seed)
    y, x = np.mgrid[0:height, 0:width].astype(np.float64)
    img = np.empty((height, width, 3), dtype=np.float64)
    u = x / max(width - 1, 1)
    v = y / max(height - 1, 1)
    for c in range(3):
        if span is None:
            img[:, :, c] = 32.0 + 1.5 * x + 1.5 * y + 20.0 * c
        else:
            # three differently oriented ramps, each spanning 0..span
            ramp = (0.5 * (u + v), 0.5 * ((1.0 - u) + v), 0.5 * (u + (1.0 - v)))[c]
            img[:, :, c] = span * ramp
    img += sigma * s.normal(height * width * 3).reshape(height, width, 3)
    return _to_u8(img)


def cosine_field(seed, width, height, sigma=6.0, terms=6):
    """Smooth low-frequency cosine field (random amplitudes, frequencies, phases) + noise."""
    s = Stream(seed)
    y, x = np.mgrid[0:height, 0:width].astype(np.float64)
    img = np.full((height, width, 3), 128.0)
    for c in range(3):
        amp = 8.0 + 16.0 * s.uniform(terms)
        fx = 0.5 + 2.5 * s.uniform(terms)
        fy = 0.5 + 2.5 * s.uniform(terms)
        ph = 2.0 * np.pi * s.uniform(terms)
        for k in range(terms):
            img[:, :, c] += amp[k] * np.cos(2.0 * np.pi * (fx[k] * x / width + fy[k] * y / height)
                                            + ph[k])
    img += sigma * s.normal(height * width * 3).reshape(height, width, 3)
    return _to_u8(img)


def voronoi_scene(seed, width, height, sites=40, sigma=3.0):
    """Piecewise-constant regions with per-region texture and 1-px dark edges."""
    s = Stream(seed)
    sx = s.uniform(sites) * width
    sy = s.uniform(sites) * height
    colours = s.integers(30, 225, sites * 3).reshape(sites, 3).astype(np.float64)
    label = np.empty((height, width), dtype=np.int32)
    xs = np.arange(width, dtype=np.float32)[None, :, None]
    rows = 64
    for y0 in range(0, height, rows):
        ys = np.arange(y0, min(y0 + rows, height), dtype=np.float32)[:, None, None]
        d = (xs - sx.astype(np.float32)[None, None, :]) ** 2 + \
            (ys - sy.astype(np.float32)[None, None, :]) ** 2
        label[y0:y0 + rows] = np.argmin(d, axis=2)
    img = colours[label] + sigma * s.normal(height * width * 3).reshape(height, width, 3)
    edge = np.zeros((height, width), dtype=bool)
    edge[:, :-1] |= label[:, :-1] != label[:, 1:]
    edge[:-1, :] |= label[:-1, :] != label[1:, :]
    out = _to_u8(img)
    out[edge] = 16
    return out


def uniform_bytes(seed, width, height):
    return Stream(seed).bytes(width * height * 3).reshape(height, width, 3)


# ---------------------------------------------------------------------------
# the five benchmark configurations

def config1():
    """Single 64x64 image: gradient + noise sigma 4."""
    return [gradient_noise(0, 64, 64, 4.0)]


def config2_shapes(n=256):
    out = []
    for k in range(n):
        s = Stream(2000 + k, lane=7)
        w = int(s.integers(400, 500)[0])
        h = int(s.integers(300, 375)[0])
        out.append((w, h))
    return out


def config2(n=256):
    """Photo-sized batch: n images, W in 400..500, H in 300..375, cosine field + noise."""
    return [cosine_field(2000 + k, w, h, 6.0) for k, (w, h) in enumerate(config2_shapes(n))]


def config3(n=32, width=2048, height=1024):
    """Street-scene-shaped batch: n images of 2048x1024, Voronoi regions."""
    return [voronoi_scene(3000 + k, width, height) for k in range(n)]


def config4(n=8, width=3840, height=2160):
    """High-resolution stress: first half compressible gradients, second half random bytes."""
    out = []
    for k in range(n):
        if k < n // 2:
            out.append(gradient_noise(4000 + k, width, height, 2.0, span=255.0))
        else:
            out.append(uniform_bytes(4000 + k, width, height))
    return out


def config5_crops(shapes, crop=224):
    """Per image: (x0, y0, flip) for a crop x crop window, seeded."""
    out = []
    for k, (w, h) in enumerate(shapes):
        s = Stream(5000 + k, lane=3)
        x0 = int(s.integers(0, w - crop)[0])
        y0 = int(s.integers(0, h - crop)[0])
        flip = int(s.uniform(1)[0] < 0.5)
        out.append((x0, y0, flip))
    return out


IMAGENET_MEAN = (0.485, 0.456, 0.406)
IMAGENET_STD = (0.229, 0.224, 0.225)
