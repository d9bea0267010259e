"""Seeded synthetic images for the five benchmark configurations.

Each generator draws from numpy's PCG64 (`default_rng`) with a fixed seed, so
the same pixels, and therefore the same JPEG bytes, come out everywhere.
Config `c` (1-based) uses seed BASE_SEED + c; image `j` of the batch config
uses BASE_SEED + 4000 + j.
"""
from __future__ import annotations

import hashlib
import os

import numpy as np

from .jpeg import EncodedJpeg, encode_jpeg

BASE_SEED = 211109219

# what each configuration is: geometry, coding parameters ("Input recipe")
CONFIGS = {
    1: dict(name="gray256_q75", width=256, height=256, ncomp=1, subsampling="gray", quality=75, optimize=False),
    2: dict(name="hd1088_444_q90", width=1920, height=1088, ncomp=3, subsampling="444", quality=90, optimize=False),
    3: dict(name="sq4096_420_q95_opt", width=4096, height=4096, ncomp=3, subsampling="420", quality=95, optimize=True),
    4: dict(name="batch256_512x384_420", width=512, height=384, ncomp=3, subsampling="420", quality=None,
            optimize=False, batch=256, qualities=(70, 80, 85, 90, 95)),
    5: dict(name="uhd16k_420_q92_flat_random", width=15360, height=8640, ncomp=3, subsampling="420", quality=92,
            optimize=False),
}


def _clip_u8(a: np.ndarray) -> np.ndarray:
    return np.clip(np.rint(a), 0, 255).astype(np.uint8)


def _gradient(rng: np.random.Generator, h: int, w: int) -> np.ndarray:
    """Per-channel linear ramps with random direction and end values, float32 [h,w,3]."""
    yy = np.linspace(0.0, 1.0, h, dtype=np.float32)[:, None]
    xx = np.linspace(0.0, 1.0, w, dtype=np.float32)[None, :]
    out = np.empty((h, w, 3), dtype=np.float32)
    for c in range(3):
        ang = rng.uniform(0, 2 * np.pi)
        lo, hi = rng.uniform(20, 235, size=2)
        t = np.cos(ang) * (xx - 0.5) + np.sin(ang) * (yy - 0.5)  # in [-0.71, 0.71]
        out[..., c] = lo + (hi - lo) * (t / 1.4143 + 0.5)
    return out


def _paint_shapes(rng: np.random.Generator, img: np.ndarray, count: int) -> None:
    """Filled axis-aligned rectangles and ellipses of random colour, position and size (in place)."""
    h, w = img.shape[:2]
    for _ in range(count):
        colour = rng.uniform(0, 255, size=3).astype(np.float32)
        cx, cy = rng.uniform(0, w), rng.uniform(0, h)
        rx, ry = rng.uniform(0.02, 0.25) * w, rng.uniform(0.02, 0.25) * h
        x0, x1 = int(max(0, cx - rx)), int(min(w, cx + rx + 1))
        y0, y1 = int(max(0, cy - ry)), int(min(h, cy + ry + 1))
        if x1 <= x0 or y1 <= y0:
            continue
        if rng.random() < 0.5:
            img[y0:y1, x0:x1] = colour
        else:
            ys = (np.arange(y0, y1, dtype=np.float32)[:, None] - cy) / ry
            xs = (np.arange(x0, x1, dtype=np.float32)[None, :] - cx) / rx
            mask = ys * ys + xs * xs <= 1.0
            img[y0:y1, x0:x1][mask] = colour


def _value_noise(rng: np.random.Generator, n: int, octaves: int) -> np.ndarray:
    """Sum of bilinearly up-sampled random lattices; octave o has 2^(o+2)+1 points per side, amplitude 2^-o."""
    acc = np.zeros((n, n), dtype=np.float32)
    pos = np.arange(n, dtype=np.float64)
    for o in range(octaves):
        m = 2 ** (o + 2) + 1
        lattice = rng.uniform(-1.0, 1.0, size=(m, m)).astype(np.float32)
        t = pos * (m - 1) / n
        i0 = np.minimum(t.astype(np.int64), m - 2)
        f = (t - i0).astype(np.float32)
        wmat = np.zeros((n, m), dtype=np.float32)  # interpolation weights, two per row
        wmat[np.arange(n), i0] = 1.0 - f
        wmat[np.arange(n), i0 + 1] = f
        acc += (wmat @ lattice @ wmat.T) * np.float32(2.0 ** -o)
    return acc


def config_image(c: int) -> np.ndarray:
    """Pixels of single-image configuration c in {1,2,3,5}: uint8 [H,W] or [H,W,3]."""
    cfg = CONFIGS[c]
    h, w = cfg["height"], cfg["width"]
    rng = np.random.default_rng(BASE_SEED + c)
    if c == 1:
        y, x = np.mgrid[0:h, 0:w].astype(np.float64)
        img = np.full((h, w), 128.0)
        for _ in range(4):
            fx, fy = rng.uniform(0.5, 4.0, size=2)
            ph = rng.uniform(0, 2 * np.pi)
            img += 60.0 * np.sin(2 * np.pi * (fx * x + fy * y) / 256.0 + ph)
        img += rng.normal(0.0, 8.0, size=(h, w))
        return _clip_u8(img)
    if c == 2:
        img = _gradient(rng, h, w)
        _paint_shapes(rng, img, 20)
        img += rng.normal(0.0, 6.0, size=(h, w, 3)).astype(np.float32)
        return _clip_u8(img)
    if c == 3:
        img = np.empty((h, w, 3), dtype=np.float32)
        for ch in range(3):
            v = _value_noise(rng, h, 8)
            v = (v - v.mean()) / max(float(np.abs(v - v.mean()).max()), 1e-6)  # span about +-1
            img[..., ch] = 128.0 + 100.0 * v
        img += rng.normal(0.0, 12.0, size=(h, w, 3)).astype(np.float32)
        return _clip_u8(img)
    if c == 5:
        half = w // 2
        img = np.empty((h, w, 3), dtype=np.uint8)
        # left half: near-flat (long end-of-block runs, short codewords)
        step = 1080
        for y0 in range(0, h, step):
            y1 = min(h, y0 + step)
            img[y0:y1, :half] = _clip_u8(128.0 + rng.standard_normal(size=(y1 - y0, half, 3), dtype=np.float32))
        # right half: uniform random pixels (long codewords)
        for y0 in range(0, h, step):
            y1 = min(h, y0 + step)
            img[y0:y1, half:] = rng.integers(0, 256, size=(y1 - y0, w - half, 3), dtype=np.uint8)
        return img
    raise ValueError("config %d is not a single-image configuration" % c)


def batch_image(j: int):
    """Image j of the batch configuration: (pixels uint8 [384,512,3], quality)."""
    cfg = CONFIGS[4]
    h, w = cfg["height"], cfg["width"]
    rng = np.random.default_rng(BASE_SEED + 4000 + j)
    quality = int(rng.choice(cfg["qualities"]))
    sigma = rng.uniform(2.0, 15.0)
    img = _gradient(rng, h, w)
    _paint_shapes(rng, img, int(rng.integers(5, 16)))
    img += rng.normal(0.0, sigma, size=(h, w, 3)).astype(np.float32)
    return _clip_u8(img), quality


def small_image(seed: int, h: int, w: int, ncomp: int = 3, sigma: float = 6.0, shapes: int = 4) -> np.ndarray:
    """A small test image of arbitrary size: gradient + shapes + noise (gray = its green channel)."""
    rng = np.random.default_rng(BASE_SEED + 100000 + seed)
    img = _gradient(rng, h, w)
    _paint_shapes(rng, img, shapes)
    img += rng.normal(0.0, sigma, size=(h, w, 3)).astype(np.float32)
    out = _clip_u8(img)
    return out if ncomp == 3 else np.ascontiguousarray(out[..., 1])


def _cache_dir():
    d = os.environ.get("JPGD_WORKLOAD_CACHE", "")
    return d or None


def config_jpeg(c: int, want_coef: bool = False, limit: int | None = None, restart_interval: int = 0,
                quality: int | None = None):
    """Encoded file(s) of configuration c: an EncodedJpeg, or for the batch config a list of them.

    `limit` truncates the batch (tests use a few images of it).  `restart_interval` (MCUs; 0 = none, as the
    configurations are defined) encodes the same pixels with restart markers; `quality` overrides the
    configuration's quality (single-image configurations only).  If JPGD_WORKLOAD_CACHE names
    a directory, files are kept there between runs, keyed by the encoder source's hash.
    """
    cfg = CONFIGS[c]
    if c == 4:
        n = cfg["batch"] if limit is None else min(limit, cfg["batch"])
        out = []
        for j in range(n):
            px, q = batch_image(j)
            out.append(encode_jpeg(px, quality=q, subsampling=cfg["subsampling"], optimize=False, want_coef=want_coef,
                                   restart_interval=restart_interval))
        return out
    cache = _cache_dir()
    path = None
    if cache and not want_coef:
        here = os.path.dirname(os.path.abspath(__file__))
        hsh = hashlib.sha256()
        for fn in ("jpeg_encoder.c", "images.py"):
            with open(os.path.join(here, fn), "rb") as f:
                hsh.update(f.read())
        tag = ("_ri%d" % restart_interval if restart_interval else "") + ("_q%d" % quality if quality else "")
        path = os.path.join(cache, "cfg%d%s_%s.npz" % (c, tag, hsh.hexdigest()[:16]))
        if os.path.exists(path):
            z = np.load(path)
            return EncodedJpeg(z["data"], None, int(z["scan_offset"]), int(z["scan_len"]), cfg["width"],
                               cfg["height"], cfg["ncomp"], cfg["subsampling"])
    enc = encode_jpeg(config_image(c), quality=quality or cfg["quality"], subsampling=cfg["subsampling"],
                      optimize=cfg["optimize"], want_coef=want_coef, restart_interval=restart_interval)
    if path:
        os.makedirs(cache, exist_ok=True)
        tmp = path + ".tmp%d.npz" % os.getpid()
        np.savez(tmp, data=enc.data, scan_offset=enc.scan_offset, scan_len=enc.scan_len)
        os.replace(tmp, path)
    return enc
