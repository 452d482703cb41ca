"""Seeded synthetic inputs for the SwitchBack layer (shapes of CLIP ViT linear layers).

This module holds NO arithmetic of the method: it only draws random matrices and rounds them to bf16.  Both the
GPU tests and the CPU oracle's tests take their inputs from here, so neither depends on a torch/numpy RNG
version.  Tensors are numpy uint16 arrays holding bf16 bit patterns.

Generator: element e of stream s under seed z is a pure function of (z, s, e) -- a splitmix64-style hash of the
counter gives two uniforms, Box-Muller (binary64) gives one standard normal, which is scaled, rounded to
binary32 and then to bf16 (round-to-nearest-even).  Being counter based, any subset of rows can be generated
without generating the rest.

The layer shapes stand in for the paper's CLIP ViT-B/16, L/14 and H/14 training workloads (Section 2.2.2; the
inner dimensions quoted in Appendix C): b = images x tokens per image, n -> m the linear layer's widths.
"""
import os
from collections import namedtuple
from concurrent.futures import ThreadPoolExecutor

import numpy as np

Layer = namedtuple("Layer", "name b n m")
Config = namedtuple("Config", "name layers x_dist dy_dist")

# (X distribution, dY distribution): "normal" = N(0, sigma^2); "outlier" = N(0,1) with 0.1% of the feature
# columns multiplied by 100; "student_t3" = sigma * t(nu=3).  W is always N(0, 1/n) (fan-in initialisation).
CONFIGS = {
    "tiny": Config("tiny", [Layer("fc", 512, 256, 1024)], ("normal", 1.0), ("normal", 1.0)),
    "vit_b16": Config("vit_b16", [Layer("fc1", 6304, 768, 3072), Layer("fc2", 6304, 3072, 768)],
                      ("normal", 1.0), ("normal", 0.1)),
    "vit_l14": Config("vit_l14", [Layer("qkv", 16448, 1024, 3072), Layer("proj", 16448, 1024, 1024),
                                  Layer("fc1", 16448, 1024, 4096), Layer("fc2", 16448, 4096, 1024)],
                      ("normal", 1.0), ("normal", 0.1)),
    "vit_h14": Config("vit_h14", [Layer("qkv", 32896, 1280, 3840), Layer("proj", 32896, 1280, 1280),
                                  Layer("fc1", 32896, 1280, 5120), Layer("fc2", 32896, 5120, 1280)],
                      ("normal", 1.0), ("normal", 0.1)),
    "outlier": Config("outlier", [Layer("up", 16384, 4096, 16384), Layer("down", 16384, 16384, 4096)],
                      ("outlier", 1.0), ("student_t3", 0.01)),
}

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 21


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_key(seed, stream):
    with np.errstate(over="ignore"):
        k = np.array([seed], dtype=np.uint64) * _GOLDEN + np.array([stream], dtype=np.uint64)
        return _mix(_mix(k) + _GOLDEN)[0]


def _uniform(key, counters):
    """Uniforms in (0,1) from 64-bit counters (53 random bits, never exactly 0 or 1)."""
    with np.errstate(over="ignore"):
        bits = _mix(_mix(counters * _GOLDEN + key))
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal_flat(seed, stream, index):
    """Standard normals (binary64) for the flat element indices `index` (uint64 array)."""
    key = _stream_key(seed, stream)
    u1 = _uniform(key, index * np.uint64(2))
    u2 = _uniform(key, index * np.uint64(2) + np.uint64(1))
    return np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)


def f32_to_bf16_bits(a):
    """binary32 array -> bf16 bit patterns (uint16), round-to-nearest-even; finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h):
    """bf16 bit patterns (uint16) -> binary32 (exact)."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _fill(fn, total, out_flat):
    """Evaluate fn(lo, hi) -> uint16 chunk over [0,total) in parallel chunks."""
    spans = [(lo, min(lo + _CHUNK, total)) for lo in range(0, total, _CHUNK)]

    def work(span):
        lo, hi = span
        out_flat[lo:hi] = fn(lo, hi)

    if len(spans) <= 1:
        for s in spans:
            work(s)
    else:
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(work, spans))


def _flat_index(rows, cols, lo, hi):
    """Global element indices (row * cols + col) of positions lo..hi of the gathered rows."""
    pos = np.arange(lo, hi, dtype=np.int64)
    r = rows[pos // cols]
    return (r * cols + pos % cols).astype(np.uint64)


def normal_bf16(nrows, ncols, sigma, seed, stream, rows=None):
    """[nrows,ncols] (or the listed rows of it) of N(0, sigma^2), rounded to bf16."""
    rows = np.arange(nrows, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty(len(rows) * ncols, np.uint16)

    def fn(lo, hi):
        z = _normal_flat(seed, stream, _flat_index(rows, ncols, lo, hi))
        return f32_to_bf16_bits((z * sigma).astype(np.float32))

    _fill(fn, out.size, out)
    return out.reshape(len(rows), ncols)


def student_t3_bf16(nrows, ncols, sigma, seed, stream, rows=None):
    """sigma * Student-t(nu=3): a normal over sqrt(chi^2_3 / 3); the chi^2_3 is the sum of a chi^2_2 variate
    (-2 ln u, from one more uniform stream) and one squared normal."""
    rows = np.arange(nrows, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty(len(rows) * ncols, np.uint16)

    def fn(lo, hi):
        idx = _flat_index(rows, ncols, lo, hi)
        z = _normal_flat(seed, stream, idx)
        chi2 = _normal_flat(seed, stream + 101, idx) ** 2 - 2.0 * np.log(_uniform(_stream_key(seed, stream + 202), idx))
        return f32_to_bf16_bits((sigma * z / np.sqrt(chi2 / 3.0)).astype(np.float32))

    _fill(fn, out.size, out)
    return out.reshape(len(rows), ncols)


def outlier_columns(ncols, seed, stream):
    """The ceil(0.1% * ncols) feature columns that carry x100 outliers (distinct, seeded)."""
    count = -(-ncols // 1000)
    key = _stream_key(seed, stream + 7)
    order = np.argsort(_uniform(key, np.arange(ncols, dtype=np.uint64)), kind="stable")
    return np.sort(order[:count])


def outlier_normal_bf16(nrows, ncols, seed, stream, rows=None):
    """N(0,1) with the outlier columns multiplied by 100 before the bf16 rounding."""
    rows = np.arange(nrows, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    cols = outlier_columns(ncols, seed, stream)
    gain = np.ones(ncols, np.float64)
    gain[cols] = 100.0
    out = np.empty(len(rows) * ncols, np.uint16)

    def fn(lo, hi):
        idx = _flat_index(rows, ncols, lo, hi)
        z = _normal_flat(seed, stream, idx)
        return f32_to_bf16_bits((z * gain[(idx % np.uint64(ncols)).astype(np.int64)]).astype(np.float32))

    _fill(fn, out.size, out)
    return out.reshape(len(rows), ncols)


def _draw(dist, nrows, ncols, seed, stream, rows):
    kind, sigma = dist
    if kind == "normal":
        return normal_bf16(nrows, ncols, sigma, seed, stream, rows)
    if kind == "student_t3":
        return student_t3_bf16(nrows, ncols, sigma, seed, stream, rows)
    if kind == "outlier":
        return outlier_normal_bf16(nrows, ncols, seed, stream, rows)
    raise ValueError(kind)


def make_layer_inputs(config, layer_index=0, seed=0, token_rows=None, which=("x", "w", "dy")):
    """Inputs of one layer of a named config: dict with x [b,n], w [m,n], dy [b,m] as bf16 bit patterns.

    token_rows, if given, restricts x and dy to those token rows (w is always whole); the values are the same
    as the corresponding rows of the full tensors.
    """
    cfg = CONFIGS[config]
    layer = cfg.layers[layer_index]
    s = seed + layer_index
    out = {}
    if "x" in which:
        out["x"] = _draw(cfg.x_dist, layer.b, layer.n, s, 1, token_rows)
    if "w" in which:
        out["w"] = normal_bf16(layer.m, layer.n, (1.0 / layer.n) ** 0.5, s, 2)
    if "dy" in which:
        out["dy"] = _draw(cfg.dy_dist, layer.b, layer.m, s, 3, token_rows)
    return out


def plant_edge_rows(x):
    """Overwrite the first rows of a bf16 matrix (>= 8 rows, >= 8 cols) with quantization edge cases and return
    the number of rows planted: an all-zero row; a row whose absmax is below 127/FLT_MAX (the scale overflows);
    a row of bf16 subnormals under an absmax just above that threshold; a tie row with absmax 254, where 1,3,5,7 scale to exact halves; a row already
    integer valued with absmax 127; a row with a negative absmax element."""
    assert x.shape[0] >= 8 and x.shape[1] >= 8
    c = x.shape[1]
    x[0, :] = 0
    tiny = np.full(c, 1e-38, np.float32)
    tiny[::2] *= -0.5
    x[1, :] = f32_to_bf16_bits(tiny)
    x[2, :] = (np.arange(c) % 0x7F + 1).astype(np.uint16)          # bf16 subnormal patterns 0x0001..0x007f
    x[2, 3] = f32_to_bf16_bits(np.array([4e-37], np.float32))[0]   # absmax just large enough for a finite scale
    tie = (np.arange(c) % 8 * 2 + 1).astype(np.float32)            # 1,3,5,...,15
    tie[1::2] *= -1.0
    tie[-1] = 254.0
    x[3, :] = f32_to_bf16_bits(tie)
    ints = ((np.arange(c) * 37) % 255 - 127).astype(np.float32)    # integers in [-127,127]
    ints[0] = 127.0
    x[4, :] = f32_to_bf16_bits(ints)
    neg = bf16_bits_to_f32(x[5, :]).copy()
    neg[c // 2] = -(np.abs(neg).max() * 2.0)
    x[5, :] = f32_to_bf16_bits(neg)
    return 6
